// sige_sparse_attn: attention for the edited query tokens only, against all cached
// keys and values (Sec. 3.2 "Extension to attention layers", Fig. "sige-attention"):
// the attention map is Nq x T instead of T x T.
//
// One wave owns 32 queries of one head and streams the keys in chunks of 32 * KT
// (64 keys for head sizes up to 96, 32 beyond; small heads keep two waves per SIMD resident);
// the next chunk's K and V rows travel from HBM to registers while the current one is
// multiplied.  All
// products run transposed so that everything belonging to a query stays in one lane
// (pair): S^T = K Q^T leaves a query's 32 logits in the registers of lanes l and
// l+32, the online softmax needs a single cross-lane exchange, the probabilities
// feed the second MFMA (O^T = V^T P^T) straight from registers because the
// contraction index may be permuted freely as long as V^T is read with the same
// permutation, and the running rescale of O^T is lane-local.  K and V chunks are
// staged in LDS once per workgroup (4 waves = 128 queries); V is transposed on the
// way in, with an XOR swizzle on 4-key groups to keep the 2-byte stores off the same
// banks.  When few queries are active the key range is split over workgroups and a
// second small kernel merges the partial (max, sum, O) triples.  Single precision has a kernel of
// its own further down (attn_f32_kernel).
#include "common.h"

#include <algorithm>
#include <type_traits>

namespace sige {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Mma16;
template <> struct Mma16<f16> {
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& c)
    {
        union { uint4 u; f16x8 v; } x, y;
        x.u = a; y.u = b;
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(x.v, y.v, c, 0, 0, 0);
    }
};
template <> struct Mma16<bf16> {
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& c)
    {
        union { uint4 u; bf16x8 v; } x, y;
        x.u = a; y.u = b;
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, y.v, c, 0, 0, 0);
    }
};

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two floats rounded to nearest even into one 32-bit pair of T (a in the low half).
template <typename T> __device__ __forceinline__ uint32_t pack2_rne(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2_rne<f16>(float a, float b)
{
    union { f16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector((f32x2){a, b}, f16x2);
    return r.u;
}
template <> __device__ __forceinline__ uint32_t pack2_rne<bf16>(float a, float b)
{
    union { bf16x2 v; uint32_t u; } r;
    r.v = __builtin_convertvector((f32x2){a, b}, bf16x2);
    return r.u;
}

struct AttnArgs {
    const void* q;
    const void* k;
    const void* v;
    void* o;
    float* ws;       // partials [split][head][Nq][d + 4] when splits > 1: the d sums, the maximum, the denominator, 2 unused
                     // (rows of whole 16-byte vectors; d is a multiple of 4)
    int q_ld, kv_ld, o_ld;
    int Nq, T, heads, d;
    int splits, chunks_per_split;
    float scale_log2e;
    // queries taken from a full tensor by block list (q_blocks != NULL): query i is pixel i % q_tpb of
    // block i / q_tpb, at row (y0 + py) * q_W + x0 + px of q (clamped into the q_H x q_W map)
    const int32_t* q_blocks;
    int q_tpb, q_bw, q_H, q_W;
};

// 32-key tiles per chunk, by head size (DT = 32-wide tiles over d)
constexpr int key_tiles(int DT) { return DT <= 3 ? 2 : 1; }
static int keys_per_chunk(int d, sige_dtype dt) { return dt == SIGE_F32 ? 32 : 32 * key_tiles((d + 31) / 32); }

// DT = 32-wide tiles over d; ODD: d takes an odd number of 16-wide steps (d % 32 is 8 or 16), so the
// last tile of V^T has spare rows.  One of them is then a row of ones: the second product sums the
// probabilities of a query - exactly the rounded values that it multiplies V with - into that row of
// O^T, the running rescale included, and the softmax spends no vector instruction on the denominator.
// The softmax is what bounds this kernel (for d = 40 its vector instructions outweigh the matrix
// instructions), so it is kept to a maximum, one fused multiply-add, one exponential and the rounding
// per logit: logits are compared raw and scaled inside the exponent, keys past T are masked only in
// the chunk that holds them, and the accumulators are rescaled only when some query's maximum moved.
template <typename T, int DT, int ODD>
__global__ __launch_bounds__(256, DT <= 3 ? 2 : 1) void attn_kernel(AttnArgs a)
{
    constexpr int KT = key_tiles(DT);
    constexpr int KCH = 32 * KT;                   // keys per chunk
    constexpr int VT_STRIDE = KCH * 2 + 8;         // bytes per row of the transposed V chunk (pad 8)
    constexpr int DKMAX = 2 * DT;                  // 16-wide steps over d for S^T, at most
    constexpr int DK = 2 * DT - ODD;               // ... and exactly
    constexpr int NV = (KT * DT + 1) / 2;          // K (and V) vectors a thread stages per chunk, at most
    extern __shared__ uint4 lds4[];
    char* lds = reinterpret_cast<char*>(lds4);
    const int d = a.d;
    const int k_stride = d * 2 + 16;               // bytes per staged K row
    char* ks = lds;                                // [KCH][k_stride]
    char* vt = lds + KCH * k_stride;               // [DT*32][VT_STRIDE]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int head = blockIdx.y;
    const int qi = (blockIdx.x * 4 + wave) * 32 + l32;
    const bool q_ok = qi < a.Nq;
    const int dvec = d / 8;                        // 16-byte vectors per row

    const int chunks_total = (a.T + KCH - 1) / KCH;
    const int c_begin = blockIdx.z * a.chunks_per_split;
    const int c_end = min(c_begin + a.chunks_per_split, chunks_total);

    // Q fragments (B operand of S^T = K Q^T): 8 consecutive d values of this lane's query
    uint4 qf[DKMAX];
    long qrow = qi;
    if (a.q_blocks != nullptr && q_ok) {
        const int b = qi / a.q_tpb, p = qi - b * a.q_tpb;
        const int py = p / a.q_bw, px = p - py * a.q_bw;
        const int y0 = a.q_blocks[2 * b], x0 = a.q_blocks[2 * b + 1];
        qrow = (long)min(max(y0 + py, 0), a.q_H - 1) * a.q_W + min(max(x0 + px, 0), a.q_W - 1);
    }
#pragma unroll
    for (int s = 0; s < DKMAX; ++s) {
        const int dd = 16 * s + 8 * half;
        qf[s] = make_uint4(0, 0, 0, 0);
        if (q_ok && dd < d)
            qf[s] = *(const uint4*)((const char*)a.q + (qrow * a.q_ld + head * d + dd) * 2);
    }
    // rows d .. DT*32 of V^T never receive data: zero them once (row d: ones, see above); likewise the
    // 16 bytes behind the d values of every staged K row, which the last 16-wide step reads when d is
    // not a multiple of 16
    constexpr uint32_t ONE2 = std::is_same<T, bf16>::value ? 0x3f803f80u : 0x3c003c00u;
    for (int j = tid; j < (DT * 32 - d) * (VT_STRIDE / 4); j += 256)
        *(uint32_t*)(vt + d * VT_STRIDE + j * 4) = (ODD && j < KCH / 2) ? ONE2 : 0u;
    for (int j = tid; j < KCH; j += 256) *(uint4*)(ks + j * k_stride + d * 2) = make_uint4(0, 0, 0, 0);

    // The vectors of a chunk this thread stages: (key, 16-byte group of d), the same for every chunk.
    int skey[NV], sdv[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int j = tid + u * 256;
        skey[u] = j < KCH * dvec ? j / dvec : -1;
        sdv[u] = j < KCH * dvec ? j - skey[u] * dvec : 0;
    }
    uint4 kreg[NV], vreg[NV];
    // HBM -> registers; keys past the end read the last key's row (a valid address) and are zeroed
    // when they are written to LDS
    auto fetch = [&](int c) {
        const int t0 = c * KCH;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (skey[u] < 0) continue;
            const long off = ((long)min(t0 + skey[u], a.T - 1) * a.kv_ld + head * d + sdv[u] * 8) * 2;
            kreg[u] = *(const uint4*)((const char*)a.k + off);
            vreg[u] = *(const uint4*)((const char*)a.v + off);
        }
    };
    // registers -> LDS: K rows as they are, V transposed
    auto commit = [&]() {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (skey[u] < 0) continue;
            const int key = skey[u], dv = sdv[u];
            // (keys past the end hold a copy of the last key's rows: their logits are masked, so their
            // probabilities are exactly zero)
            const uint4 kv = kreg[u], vv = vreg[u];
            *(uint4*)(ks + key * k_stride + dv * 16) = kv;
            // element e of this vector is row dv*8+e of V^T; the index of the 4-key group is swizzled
            // by dv in its low three bits
            const int col = ((((key >> 2) ^ (dv & 7)) << 2) | (key & 3)) * 2;
            union { uint4 u4; uint16_t h[8]; } x;
            x.u4 = vv;
#pragma unroll
            for (int e = 0; e < 8; ++e) *(uint16_t*)(vt + (dv * 8 + e) * VT_STRIDE + col) = x.h[e];
        }
    };

    f32x16 oacc[DT];
#pragma unroll
    for (int nt = 0; nt < DT; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[nt][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    if (c_begin < c_end) fetch(c_begin);
    for (int c = c_begin; c < c_end; ++c) {
        const int t0 = c * KCH;
        __syncthreads();  // previous chunk fully consumed
        commit();
        __syncthreads();
        if (c + 1 < c_end) fetch(c + 1);          // in flight while this chunk is multiplied
        __builtin_amdgcn_sched_barrier(0);        // (kept above the MFMAs: the scheduler would sink the loads)

        // S^T chunk: rows = keys (KT tiles of 32), cols = queries
        f32x16 sacc[KT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kt][r] = 0.0f;
            // all K fragments of the tile first (independent LDS reads, one latency), then the MFMAs:
            // read one by one, each in front of its MFMA, they cost a round trip to LDS per step
            uint4 kf[DK];
#pragma unroll
            for (int s = 0; s < DK; ++s)
                kf[s] = *(const uint4*)(ks + (kt * 32 + l32) * k_stride + (16 * s + 8 * half) * 2);
#pragma unroll
            for (int s = 0; s < DK; ++s) Mma16<T>::run(kf[s], qf[s], sacc[kt]);
        }
        // online softmax; of tile kt this lane holds keys 8*(r/4) + 4*half + r%4 of its query
        if (t0 + KCH > a.T) {                      // the chunk that holds the end of the keys
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = t0 + kt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (key >= a.T) sacc[kt][r] = -INFINITY;
                }
        }
        float mr = sacc[0][0];                     // raw logits: the scale (>= 0) goes into the exponent
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mr = fmaxf(mr, sacc[kt][r]);
        mr = fmaxf(mr, __shfl_xor(mr, 32));
        const float mx = fmaxf(m_run, mr * a.scale_log2e);
        if (__builtin_amdgcn_ballot_w64(mx != m_run) != 0ull) {     // some query's maximum moved
            const float alpha = __builtin_amdgcn_exp2f(m_run - mx);  // first chunk: exp2(-inf) = 0
            m_run = mx;
            l_run *= alpha;
#pragma unroll
            for (int nt = 0; nt < DT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[nt][r] *= alpha;
        }
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                sacc[kt][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt][r], a.scale_log2e, -m_run));

        // O^T += V^T P^T, two steps of 16 keys per tile; step s uses registers 8s..8s+7.
        // The probabilities enter this product in the storage type.  fp16 keeps 11 bits of a
        // probability; bf16 keeps 8, too few for the stated tolerance on rows spread over many keys,
        // so there a probability goes in as the sum of two bf16 numbers (the rounded value and the
        // rounded remainder, 16 bits together) and the same V^T fragments are multiplied twice.
        // The row's denominator sums what the product multiplies with: through the row of ones (ODD),
        // else here - the rounded fp16 values, or for bf16 the unrounded ones (which the two terms
        // match to 2^-16) - so that numerator and denominator carry the same rounding and a row
        // dominated by one key returns that key's value row.  With the row of ones fp16 may even
        // truncate (one instruction per pair): the truncation is in both.
        constexpr bool TWO = std::is_same<T, bf16>::value;
        float lsum = 0.0f;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                uint32_t ph[4], pl[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p0 = sacc[kt][8 * s + 2 * j], p1 = sacc[kt][8 * s + 2 * j + 1];
                    if constexpr (TWO) {
                        ph[j] = pack2_rne<T>(p0, p1);
                        const float h0 = __uint_as_float(ph[j] << 16), h1 = __uint_as_float(ph[j] & 0xffff0000u);
                        pl[j] = pack2_rne<T>(p0 - h0, p1 - h1);
                        if constexpr (!ODD) lsum += p0 + p1;
                    } else if constexpr (ODD) {
                        union { decltype(__builtin_amdgcn_cvt_pkrtz(0.f, 0.f)) v; uint32_t u; } r;
                        r.v = __builtin_amdgcn_cvt_pkrtz(p0, p1);
                        ph[j] = r.u;
                    } else {
                        union { f16x2 v; uint32_t u; } r;
                        r.u = ph[j] = pack2_rne<T>(p0, p1);
                        lsum += (float)r.v.x + (float)r.v.y;
                    }
                }
                const uint4 pf = make_uint4(ph[0], ph[1], ph[2], ph[3]);
                uint2 lo[DT], hi[DT];                        // likewise: the V^T fragments of all tiles, then the MFMAs
#pragma unroll
                for (int nt = 0; nt < DT; ++nt) {
                    const int row = nt * 32 + l32;
                    const int sw = (row >> 3) & 7;
                    const int g_lo = kt * 8 + ((4 * s + half) ^ sw), g_hi = kt * 8 + ((4 * s + 2 + half) ^ sw);
                    lo[nt] = *(const uint2*)(vt + row * VT_STRIDE + g_lo * 8);
                    hi[nt] = *(const uint2*)(vt + row * VT_STRIDE + g_hi * 8);
                }
#pragma unroll
                for (int nt = 0; nt < DT; ++nt) {
                    const uint4 vf = make_uint4(lo[nt].x, lo[nt].y, hi[nt].x, hi[nt].y);
                    Mma16<T>::run(vf, pf, oacc[nt]);
                    if constexpr (TWO) Mma16<T>::run(vf, make_uint4(pl[0], pl[1], pl[2], pl[3]), oacc[nt]);
                }
            }
        l_run += lsum;
    }

    float l_tot;
    if constexpr (ODD) {
        // row d of O^T (in the last tile: row 8 or 16, held by the lower half of the wave in register 4 or 8)
        const float ones = (d & 31) == 8 ? oacc[DT - 1][4] : oacc[DT - 1][8];
        l_tot = __shfl(ones, l32);
    } else {
        l_tot = l_run + __shfl_xor(l_run, 32);
    }
    if (!q_ok) return;
    if (a.splits == 1) {
        const float inv = 1.0f / l_tot;
#pragma unroll
        for (int nt = 0; nt < DT; ++nt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dd = nt * 32 + 8 * rq + 4 * half;
                if (dd < d) {
                    union { uint2 u; T h[4]; } x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x.h[e] = from_f32<T>(oacc[nt][4 * rq + e] * inv);
                    *(uint2*)((char*)a.o + ((long)qi * a.o_ld + head * d + dd) * 2) = x.u;
                }
            }
    } else {
        float* w = a.ws + (((long)blockIdx.z * a.heads + head) * a.Nq + qi) * (d + 4);
        if (half == 0) *(float2*)(w + d) = make_float2(m_run, l_tot);
#pragma unroll
        for (int nt = 0; nt < DT; ++nt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dd = nt * 32 + 8 * rq + 4 * half;
                if (dd < d)
                    *(float4*)(w + dd) = make_float4(oacc[nt][4 * rq], oacc[nt][4 * rq + 1], oacc[nt][4 * rq + 2],
                                                     oacc[nt][4 * rq + 3]);
            }
    }
}

// Single precision (the precision the paper's experiments run in, Sec. 4.1 "Implementation details"):
// the same transposed products on v_mfma_f32_32x32x2_f32, whose operands are one value per lane, so
// nothing is rounded between the two products and V needs no transpose (a lane picks V[key][d]
// itself).  A workgroup of NW waves holds its 32 * NW query rows in LDS (row stride d + 1 words, so
// that the lanes of a half fall on different banks) and stages 32 keys per chunk.
template <int DT, int NW>
__global__ __launch_bounds__(64 * NW) void attn_f32_kernel(AttnArgs a)
{
    constexpr int NT = 64 * NW;
    constexpr int KCH = 32;
    constexpr int VS = DT * 32 + 4;                // words per staged V row (columns d .. DT*32 stay zero)
    constexpr int NV = (8 * DT * 32 + NT - 1) / NT; // 16-byte vectors of K (and of V) a thread stages per chunk, at most
    extern __shared__ uint4 lds4[];
    float* lds = reinterpret_cast<float*>(lds4);
    const int d = a.d;
    const int rs = d + 1;                          // words per staged Q or K row
    float* qsm = lds;                              // [NW*32][rs]
    float* ksm = qsm + NW * 32 * rs;               // [KCH][rs]
    float* vsm = ksm + KCH * rs;                   // [KCH][VS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int head = blockIdx.y;
    const int q0 = blockIdx.x * (NW * 32);
    const int qi = q0 + wave * 32 + l32;
    const bool q_ok = qi < a.Nq;
    const int dvec = d / 4;

    const int chunks_total = (a.T + KCH - 1) / KCH;
    const int c_begin = blockIdx.z * a.chunks_per_split;
    const int c_end = min(c_begin + a.chunks_per_split, chunks_total);

    // the workgroup's query rows (rows past Nq are zero)
    for (int j = tid; j < NW * 32 * dvec; j += NT) {
        const int row = j / dvec, dv = j - row * dvec;
        const int qq = q0 + row;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (qq < a.Nq) {
            long qrow = qq;
            if (a.q_blocks != nullptr) {
                const int b = qq / a.q_tpb, p = qq - b * a.q_tpb;
                const int py = p / a.q_bw, px = p - py * a.q_bw;
                const int y0 = a.q_blocks[2 * b], x0 = a.q_blocks[2 * b + 1];
                qrow = (long)min(max(y0 + py, 0), a.q_H - 1) * a.q_W + min(max(x0 + px, 0), a.q_W - 1);
            }
            v = *(const float4*)((const float*)a.q + qrow * a.q_ld + head * d + dv * 4);
        }
        float* dst = qsm + row * rs + dv * 4;
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    for (int j = tid; j < KCH * (VS - d); j += NT) {
        const int key = j / (VS - d), c = j - key * (VS - d);
        vsm[key * VS + d + c] = 0.0f;
    }

    int skey[NV], sdv[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int j = tid + u * NT;
        skey[u] = j < KCH * dvec ? j / dvec : -1;
        sdv[u] = j < KCH * dvec ? j - skey[u] * dvec : 0;
    }
    float4 kreg[NV], vreg[NV];
    auto fetch = [&](int c) {
        const int t0 = c * KCH;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (skey[u] < 0) continue;
            const long off = (long)min(t0 + skey[u], a.T - 1) * a.kv_ld + head * d + sdv[u] * 4;
            kreg[u] = *(const float4*)((const float*)a.k + off);
            vreg[u] = *(const float4*)((const float*)a.v + off);
        }
    };
    auto commit = [&](int c) {
        const int t0 = c * KCH;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (skey[u] < 0) continue;
            const bool in = t0 + skey[u] < a.T;
            const float4 kv = in ? kreg[u] : make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 vv = in ? vreg[u] : make_float4(0.f, 0.f, 0.f, 0.f);
            float* kd = ksm + skey[u] * rs + sdv[u] * 4;
            kd[0] = kv.x; kd[1] = kv.y; kd[2] = kv.z; kd[3] = kv.w;
            *(float4*)(vsm + skey[u] * VS + sdv[u] * 4) = vv;
        }
    };

    f32x16 oacc[DT];
#pragma unroll
    for (int nt = 0; nt < DT; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[nt][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float* qrow_s = qsm + (wave * 32 + l32) * rs + half;
    const float* krow_s = ksm + l32 * rs + half;

    if (c_begin < c_end) fetch(c_begin);
    for (int c = c_begin; c < c_end; ++c) {
        const int t0 = c * KCH;
        __syncthreads();  // previous chunk fully consumed (and, the first time, the query rows written)
        commit(c);
        __syncthreads();
        if (c + 1 < c_end) fetch(c + 1);

        // S^T tile: rows = the chunk's 32 keys, cols = this wave's 32 queries; two values of d per MFMA
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.0f;
        for (int j = 0; j < d; j += 4) {              // d is a multiple of 4
            const float k0 = krow_s[j], q0v = qrow_s[j], k1 = krow_s[j + 2], q1v = qrow_s[j + 2];
            sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(k0, q0v, sacc, 0, 0, 0);
            sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(k1, q1v, sacc, 0, 0, 0);
        }
        // online softmax; this lane holds keys 8*(r/4) + 4*half + r%4 of its query
        float mx = m_run;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = t0 + 8 * (r >> 2) + 4 * half + (r & 3);
            sacc[r] = key < a.T ? sacc[r] * a.scale_log2e : -INFINITY;
            mx = fmaxf(mx, sacc[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float alpha = exp2f(m_run - mx);
        float lsum = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sacc[r] = exp2f(sacc[r] - mx);
            lsum += sacc[r];
        }
        l_run = l_run * alpha + lsum;
        m_run = mx;
#pragma unroll
        for (int nt = 0; nt < DT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[nt][r] *= alpha;
        // O^T += V^T P^T: register r of the two lane halves is one pair of keys
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float* vrow = vsm + (8 * (r >> 2) + 4 * half + (r & 3)) * VS + l32;
#pragma unroll
            for (int nt = 0; nt < DT; ++nt)
                oacc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(vrow[nt * 32], sacc[r], oacc[nt], 0, 0, 0);
        }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!q_ok) return;
    if (a.splits == 1) {
        const float inv = 1.0f / l_tot;
#pragma unroll
        for (int nt = 0; nt < DT; ++nt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dd = nt * 32 + 8 * rq + 4 * half;
                if (dd < d)
                    *(float4*)((float*)a.o + (long)qi * a.o_ld + head * d + dd) =
                        make_float4(oacc[nt][4 * rq] * inv, oacc[nt][4 * rq + 1] * inv, oacc[nt][4 * rq + 2] * inv,
                                    oacc[nt][4 * rq + 3] * inv);
            }
    } else {
        float* w = a.ws + (((long)blockIdx.z * a.heads + head) * a.Nq + qi) * (d + 4);
        if (half == 0) *(float2*)(w + d) = make_float2(m_run, l_tot);
#pragma unroll
        for (int nt = 0; nt < DT; ++nt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int dd = nt * 32 + 8 * rq + 4 * half;
                if (dd < d)
                    *(float4*)(w + dd) = make_float4(oacc[nt][4 * rq], oacc[nt][4 * rq + 1], oacc[nt][4 * rq + 2],
                                                     oacc[nt][4 * rq + 3]);
            }
    }
}

// Merge of the per-split partials.  P neighbouring lanes share one (query, head, four consecutive d
// elements): lane p takes splits p, p + P, p + 2P, p + 3P - all of its loads are in flight together, one
// round trip to memory however many splits there are - and the P partial (maximum, denominator, sums)
// triples are combined with a butterfly of lane exchanges, each step rescaling to the common maximum as
// the attention kernel does.  The order of the sums is fixed by (P, splits): results are reproducible.
template <typename T, int P>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a)
{
    constexpr int B = 4;                           // splits per lane, at most (the host picks P accordingly)
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int d = a.d, dq = d >> 2;
    const long grp = i / P;
    const int sub = (int)(i % P);
    const bool live = grp < (long)a.Nq * a.heads * dq;      // (whole groups: P divides the workgroup size)
    const long g = live ? grp : 0;
    const int dd = (int)(g % dq) * 4;
    const int head = (int)((g / dq) % a.heads);
    const int qi = (int)(g / ((long)dq * a.heads));
    const long sstride = (long)a.heads * a.Nq * (d + 4);
    const float* w0 = a.ws + ((long)head * a.Nq + qi) * (d + 4);
    float2 ml[B];
    float4 val[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const float* w = w0 + min(sub + j * P, a.splits - 1) * sstride;
        ml[j] = *(const float2*)(w + d);
        val[j] = *(const float4*)(w + dd);
    }
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < B; ++j)
        if (sub + j * P < a.splits) m = fmaxf(m, ml[j].x);
    float den = 0.0f, num[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const float f = sub + j * P < a.splits ? exp2f(ml[j].x - m) : 0.0f;
        num[0] += val[j].x * f; num[1] += val[j].y * f; num[2] += val[j].z * f; num[3] += val[j].w * f;
        den += ml[j].y * f;
    }
#pragma unroll
    for (int x = 1; x < P; x <<= 1) {
        const float m2 = __shfl_xor(m, x), den2 = __shfl_xor(den, x);
        float n2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) n2[e] = __shfl_xor(num[e], x);
        const float mm = fmaxf(m, m2);
        // a lane without splits carries (-inf, 0, 0): its weight is 0, not exp2(-inf + inf)
        const float f1 = m == -INFINITY ? 0.0f : exp2f(m - mm), f2 = m2 == -INFINITY ? 0.0f : exp2f(m2 - mm);
        // both partners add in the same order (lower lane's share first), so they hold the same bits
        const bool low = (sub & x) == 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) num[e] = low ? num[e] * f1 + n2[e] * f2 : n2[e] * f2 + num[e] * f1;
        den = low ? den * f1 + den2 * f2 : den2 * f2 + den * f1;
        m = mm;
    }
    if (!live || sub != 0) return;
    T* o = (T*)a.o + (long)qi * a.o_ld + head * d + dd;
    const float inv = 1.0f / den;
    if constexpr (sizeof(T) == 4) {
        *(float4*)o = make_float4(num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv);
    } else {
        union { uint2 u; T h[4]; } x;
#pragma unroll
        for (int e = 0; e < 4; ++e) x.h[e] = from_f32<T>(num[e] * inv);
        *(uint2*)o = x.u;
    }
}

template <typename T>
static int launch_merge(const AttnArgs& a, hipStream_t st)
{
    const long groups = (long)a.Nq * a.heads * (a.d / 4);
    auto go = [&](auto kern, int P) {
        hipLaunchKernelGGL(kern, dim3((int)((groups * P + 255) / 256)), dim3(256), 0, st, a);
    };
    if (a.splits <= 4) go(attn_merge_kernel<T, 1>, 1);
    else if (a.splits <= 16) go(attn_merge_kernel<T, 4>, 4);
    else go(attn_merge_kernel<T, 16>, 16);          // at most 64 splits
    SIGE_LAUNCH_CHECK("sige_sparse_attn(merge)");
    return SIGE_OK;
}

// Number of key splits: a workgroup walks through its key chunks one after the other and each costs
// a staging round trip, so few queries are spread over about two workgroups per compute unit (more
// splits cost the merge kernel more than they save: measured at 64 to 1280 queries), at least 2
// chunks each.
static int pick_splits(int Nq, int T, int heads, int d, sige_dtype dt)
{
    const int KCH = keys_per_chunk(d, dt);
    const long base = (long)heads * ((Nq + 127) / 128);
    const int chunks = (T + KCH - 1) / KCH;
    const int target = knob(SIGE_KNOB_ATTN_WGS);            // workgroups to aim for
    long want = ((target >= 0 ? target : 512) + base - 1) / base;
    long cap = chunks / 2;
    if (want > cap) want = cap;
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    const int per = (int)((chunks + want - 1) / want);
    return (chunks + per - 1) / per;
}

template <typename T, int DT>
static int launch_attn_dt(const AttnArgs& a, hipStream_t st)
{
    constexpr int KCH = 32 * key_tiles(DT);
    const size_t lds = (size_t)KCH * (a.d * 2 + 16) + (size_t)DT * 32 * (KCH * 2 + 8);
    dim3 grid((a.Nq + 127) / 128, a.heads, a.splits);
    const bool odd = ((a.d + 15) / 16) & 1;        // d % 32 is 8 or 16
    auto kern = odd ? attn_kernel<T, DT, 1> : attn_kernel<T, DT, 0>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "sige_sparse_attn: cannot reserve %zu bytes of LDS: %s", lds,
                     hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, a);
    SIGE_LAUNCH_CHECK("sige_sparse_attn");
    if (a.splits > 1) return launch_merge<T>(a, st);
    return SIGE_OK;
}

template <typename T>
static int launch_attn(const AttnArgs& a, hipStream_t st)
{
    const int dt = (a.d + 31) / 32;
    switch (dt) {
    case 1: return launch_attn_dt<T, 1>(a, st);
    case 2: return launch_attn_dt<T, 2>(a, st);
    case 3: return launch_attn_dt<T, 3>(a, st);
    case 4: return launch_attn_dt<T, 4>(a, st);
    case 5: return launch_attn_dt<T, 5>(a, st);
    case 6: return launch_attn_dt<T, 6>(a, st);
    default: return launch_attn_dt<T, 8>(a, st);
    }
}

template <int DT, int NW>
static int launch_attn_f32_as(const AttnArgs& a, hipStream_t st)
{
    const size_t lds = ((size_t)(NW * 32 + 32) * (a.d + 1) + 32 * (DT * 32 + 4)) * sizeof(float);
    dim3 grid((a.Nq + NW * 32 - 1) / (NW * 32), a.heads, a.splits);
    auto kern = attn_f32_kernel<DT, NW>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "sige_sparse_attn: cannot reserve %zu bytes of LDS: %s", lds,
                     hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, grid, dim3(64 * NW), lds, st, a);
    SIGE_LAUNCH_CHECK("sige_sparse_attn");
    if (a.splits > 1) return launch_merge<float>(a, st);
    return SIGE_OK;
}

// Four waves (128 queries) per workgroup while their rows, the key chunk and the value chunk fit
// the LDS of a compute unit, two beyond (heads wider than 128).
static int launch_attn_f32(const AttnArgs& a, hipStream_t st)
{
    switch ((a.d + 31) / 32) {
    case 1: return launch_attn_f32_as<1, 4>(a, st);
    case 2: return launch_attn_f32_as<2, 4>(a, st);
    case 3: return launch_attn_f32_as<3, 4>(a, st);
    case 4: return launch_attn_f32_as<4, 4>(a, st);
    case 5: return launch_attn_f32_as<5, 2>(a, st);
    case 6: return launch_attn_f32_as<6, 2>(a, st);
    default: return launch_attn_f32_as<8, 2>(a, st);
    }
}

}  // namespace sige

using namespace sige;

extern "C" size_t sige_sparse_attn_workspace_bytes(int32_t Nq, int32_t T, int32_t heads, int32_t d)
{
    if (Nq <= 0 || T <= 0 || heads <= 0 || d <= 0) return 0;
    // the larger of what the half-precision and the single-precision kernels would use
    const int splits = std::max(pick_splits(Nq, T, heads, d, SIGE_F16), pick_splits(Nq, T, heads, d, SIGE_F32));
    if (splits <= 1) return 0;
    return (size_t)splits * heads * Nq * (d + 4) * sizeof(float);
}

static int attn_entry(const char* who, AttnArgs& a, const void* q, int32_t q_ld, const void* k, const void* v,
                      int32_t kv_ld, sige_dtype dt, int32_t Nq, int32_t T, int32_t heads, int32_t d, float scale,
                      void* o, int32_t o_ld, void* workspace, size_t workspace_bytes, void* stream)
{
    SIGE_REQUIRE(Nq >= 0 && T > 0 && heads > 0 && d > 0, SIGE_ERR_INVALID_ARG,
                 "%s: need Nq >= 0, T > 0, heads > 0, d > 0", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    const int vw = dt == SIGE_F32 ? 4 : 8;                  // elements per 16-byte vector
    SIGE_REQUIRE(d % vw == 0 && d <= 256, SIGE_ERR_UNSUPPORTED, "%s: d must be a multiple of %d and <= 256", who, vw);
    SIGE_REQUIRE(heads <= 65535, SIGE_ERR_UNSUPPORTED, "%s: too many heads", who);
    if (Nq == 0) return SIGE_OK;
    SIGE_REQUIRE(q && k && v && o, SIGE_ERR_INVALID_ARG, "%s: q, k, v and o are required", who);
    SIGE_REQUIRE(q_ld >= heads * d && kv_ld >= heads * d && o_ld >= heads * d, SIGE_ERR_INVALID_ARG,
                 "%s: row strides must be >= heads*d", who);
    SIGE_REQUIRE(q_ld % vw == 0 && kv_ld % vw == 0 && o_ld % vw == 0, SIGE_ERR_UNSUPPORTED,
                 "%s: row strides must be multiples of %d elements", who, vw);
    SIGE_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(o), SIGE_ERR_UNSUPPORTED,
                 "%s: pointers must be 16-byte aligned", who);
    a.q = q; a.k = k; a.v = v; a.o = o; a.ws = (float*)workspace;
    a.q_ld = q_ld; a.kv_ld = kv_ld; a.o_ld = o_ld;
    a.Nq = Nq; a.T = T; a.heads = heads; a.d = d;
    SIGE_REQUIRE(scale >= 0.0f, SIGE_ERR_UNSUPPORTED, "%s: the scale must not be negative", who);
    a.scale_log2e = scale * 1.4426950408889634f;
    const int KCH = keys_per_chunk(d, dt);
    const int chunks = (T + KCH - 1) / KCH;
    int splits = pick_splits(Nq, T, heads, d, dt);
    if (splits > 1 && (workspace == nullptr ||
                       workspace_bytes < (size_t)splits * heads * Nq * (d + 4) * sizeof(float) ||
                       (reinterpret_cast<uintptr_t>(workspace) & 15u)))
        splits = 1;
    a.chunks_per_split = (chunks + splits - 1) / splits;
    a.splits = (chunks + a.chunks_per_split - 1) / a.chunks_per_split;
    hipStream_t st = (hipStream_t)stream;
    if (dt == SIGE_F32) return launch_attn_f32(a, st);
    return dt == SIGE_F16 ? launch_attn<f16>(a, st) : launch_attn<bf16>(a, st);
}

extern "C" int sige_sparse_attn(const void* q, int32_t q_ld, const void* k, const void* v, int32_t kv_ld,
                                sige_dtype dt, int32_t Nq, int32_t T, int32_t heads, int32_t d,
                                float scale, void* o, int32_t o_ld, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    clear_error();
    AttnArgs a;
    a.q_blocks = nullptr;
    a.q_tpb = a.q_bw = a.q_H = a.q_W = 1;
    return attn_entry("sige_sparse_attn", a, q, q_ld, k, v, kv_ld, dt, Nq, T, heads, d, scale, o, o_ld, workspace,
                      workspace_bytes, stream);
}

extern "C" int sige_sparse_attn_blocks(const void* q, int32_t q_ld, const sige_geom* g, const int32_t* indices,
                                       int32_t n_blocks, const void* k, const void* v, int32_t kv_ld,
                                       sige_dtype dt, int32_t T, int32_t heads, int32_t d, float scale, void* o,
                                       int32_t o_ld, void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    const char* who = "sige_sparse_attn_blocks";
    SIGE_REQUIRE(g != nullptr, SIGE_ERR_INVALID_ARG, "%s: geometry is required", who);
    SIGE_REQUIRE(g->k == 1 && g->stride == 1 && g->pad == 0 && g->block_h > 0 && g->block_w > 0 && g->H_in > 0 &&
                     g->W_in > 0,
                 SIGE_ERR_UNSUPPORTED, "%s: the geometry must be that of a 1x1, stride-1, unpadded layer", who);
    SIGE_REQUIRE(n_blocks >= 0, SIGE_ERR_INVALID_ARG, "%s: n_blocks must be a host value >= 0", who);
    SIGE_REQUIRE((long)n_blocks * g->block_h * g->block_w <= 0x7fffffffL, SIGE_ERR_UNSUPPORTED,
                 "%s: too many query rows", who);
    if (n_blocks == 0) return SIGE_OK;
    SIGE_REQUIRE(indices != nullptr, SIGE_ERR_INVALID_ARG, "%s: indices are required", who);
    AttnArgs a;
    a.q_blocks = indices;
    a.q_tpb = g->block_h * g->block_w;
    a.q_bw = g->block_w;
    a.q_H = g->H_in;
    a.q_W = g->W_in;
    return attn_entry(who, a, q, q_ld, k, v, kv_ld, dt, n_blocks * a.q_tpb, T, heads, d, scale, o, o_ld, workspace,
                      workspace_bytes, stream);
}
