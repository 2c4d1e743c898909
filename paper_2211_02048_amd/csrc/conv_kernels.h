// The convolution kernels and their launchers (templates over the storage type).  Included by the
// three translation units that instantiate them, one per storage type, and by conv.hip, which holds
// the planning and the entry points and only declares the instantiations.
#pragma once
#include <type_traits>

#include "common.h"

#include <algorithm>

namespace sige {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One 16-byte A fragment and one 16-byte B fragment per lane advance K by KSTEP channels.
template <typename T> struct Mma;
template <> struct Mma<f16> {
    static constexpr int KSTEP = 16;
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& c)
    {
        union { uint4 u; f16x8 v; } x, y;
        x.u = a; y.u = b;
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(x.v, y.v, c, 0, 0, 0);
    }
};
template <> struct Mma<bf16> {
    static constexpr int KSTEP = 16;
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& c)
    {
        union { uint4 u; bf16x8 v; } x, y;
        x.u = a; y.u = b;
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, y.v, c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    static constexpr int KSTEP = 8;  // lane half h holds channels 4h..4h+3 of the step
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x16& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

struct ConvArgs {
    const void* tiles;
    const void* w;
    const float* bias;
    void* out;
    const int32_t* count;
    int th, tw, bh, bw, k, stride, Cin, Cout;
    int max_blocks, n_host;
    int G;      // whole blocks per workgroup (1 when a block is split into row bands)
    int rows;   // output rows of a block handled by one workgroup
    int trows;  // tile rows staged: (rows-1)*stride + k
    int Cc;     // channels staged per pass (multiple of KSTEP)
    int ps;     // LDS pixel stride in bytes: Cc*size + 16 (the pad spreads pixels over banks)
    // gather folded in (x != nullptr): tiles are gathered from x on the way into LDS; scatter folded
    // in (y != nullptr, indices given): the output goes to the blocks' places in y, residuals added;
    // otherwise it is stored as tiles in out
    const void* x;
    const int32_t* indices;
    const float* scale;
    const float* shift;
    const void* res_tiles;
    const void* res_full;
    void* y;
    int Hin, Win, x_ld, up, pad, act, Hout, Wout, y_ld, res_ld;
    // K split over workgroups (ksplit > 1): workgroup (band, split) multiplies only its share of
    // the channel chunks and stores fp32 partial sums, partial[split][tile element]; a second
    // kernel adds the shares in a fixed order and finishes the output
    float* partial;
    long partial_stride;
    int ksplit, bands;
    // activated copies of the output (scatter mode only): copy j receives
    // act_j(scale_j[o] * v + shift_j[o]) of every value v stored to y, at the same pixel
    struct ActOut { void* y; const float* scale; const float* shift; int ld, act; };
    ActOut ao[SIGE_MAX_ACT_OUTS];
    int n_ao;
    // gated GELU folded into the epilogue (tiles out only): the Cout convolution channels come in
    // groups of 16 = 8 values followed by their 8 gates; out has Cout / 2 channels
    int glu;
    int stagger;  // 128 x 128 shape, many rounds of workgroups: every other workgroup of the first round starts late (units of sleep)
    int direct;   // shapes with swapped operands: accumulators leave straight from the registers (else through LDS)
    // Marked mode (conv_pair_kernel only): the block list is not given but built by every workgroup
    // from the per-block flags that the marking pass left (mk_nb of them, mk_nbx per block row); the
    // call's first workgroup also stores the ordered list and its length where a compaction pass
    // would have.  `indices` is then non-null but not read.  mk_flags is the list's flag workspace:
    // two halves of mk_half bytes, then the phase words (see reduce_mask.hip).
    uint8_t* mk_flags;
    int32_t* mk_indices;
    int32_t* mk_count;
    int mk_nb, mk_nbx, mk_half;
    // divisors the kernels divide by, prepared on the host: rows * bw (a workgroup's rows per block),
    // bw, trows * tw, tw, bh * bw, and the 16-byte runs per output pixel (the reduction kernel's)
    FastDiv d_pb, d_bw, d_per, d_tw, d_pbfull, d_runs;
    FastDiv d_bands, d_ksplit, d_mk_nbx;   // bands, ksplit and (marked mode) blocks per block row
};

// Packed weight: [Cout_pad/32][k*k][Cin/KSTEP][64 lanes][16 bytes]; lane l of a fragment
// holds output channel nt*32 + l%32 and the l/32-th half of the step's channels.
template <typename T>
__global__ __launch_bounds__(256) void pack_weight_kernel(const T* __restrict__ w, int Cout, int Cin,
                                                          int k, long n_elems, T* __restrict__ packed)
{
    constexpr int N = Vec16<T>::N, KS = Mma<T>::KSTEP;
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_elems) return;
    const int e = (int)(i % N);
    const int lane = (int)((i / N) % 64);
    long r = i / (N * 64);
    const int kc = (int)(r % (Cin / KS));
    r /= (Cin / KS);
    const int tap = (int)(r % (k * k));
    const int nt = (int)(r / (k * k));
    const int o = nt * 32 + (lane & 31);
    const int c = kc * KS + (lane >> 5) * N + e;
    const int ky = tap / k, kx = tap - ky * k;
    packed[i] = o < Cout ? w[(((long)o * Cin + c) * k + ky) * k + kx] : from_f32<T>(0.0f);
}

// Finishes one run of N consecutive output channels starting at o: v holds the fp32 sums (bias
// included), t the element's index in the stacked output tiles, pix the pixel of y it belongs to.
// Plain mode stores the tile elements; fused mode adds the residuals to the fp32 sums and rounds
// once into y (Scatter with Block Residual, App. A.2: the layer's stored output is the convolution
// plus its residuals; no tile is stored on the way, so none is rounded).
// early: the two residual vectors were fetched by the caller ahead of time (for the 16-byte path
// only).
// Scale and shift of the activated copies for the N channels from o on, fetched by the caller
// ahead of the sums so that their latency does not sit behind the store of y.
template <int N> struct ActParams { float sc[SIGE_MAX_ACT_OUTS][N], sh[SIGE_MAX_ACT_OUTS][N]; };
template <int N>
__device__ __forceinline__ void load_act_params(const ConvArgs& a, int o, ActParams<N>& p)
{
#pragma unroll
    for (int j = 0; j < SIGE_MAX_ACT_OUTS; ++j) {
        if (j >= a.n_ao) break;
#pragma unroll
        for (int i = 0; i < N; ++i) { p.sc[j][i] = 1.0f; p.sh[j][i] = 0.0f; }
        if (a.ao[j].scale == nullptr) continue;
        if (aligned16_dev(a.ao[j].scale) && aligned16_dev(a.ao[j].shift)) {    // o is a multiple of N: whole vectors
#pragma unroll
            for (int i = 0; i < N / 4; ++i) {
                const f32x4 c = *(const f32x4*)(a.ao[j].scale + o + 4 * i), h = *(const f32x4*)(a.ao[j].shift + o + 4 * i);
                p.sc[j][4 * i] = c.x; p.sc[j][4 * i + 1] = c.y; p.sc[j][4 * i + 2] = c.z; p.sc[j][4 * i + 3] = c.w;
                p.sh[j][4 * i] = h.x; p.sh[j][4 * i + 1] = h.y; p.sh[j][4 * i + 2] = h.z; p.sh[j][4 * i + 3] = h.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                p.sc[j][i] = a.ao[j].scale[o + i];
                p.sh[j][i] = a.ao[j].shift[o + i];
            }
        }
    }
}

// The bias of the N channels from o on: as 16-byte vectors when the run is whole and the array is
// 16-byte aligned (o is a multiple of N), element by element otherwise; 0 where there is none.
template <int N>
__device__ __forceinline__ void load_bias(const ConvArgs& a, int o, float (&bv)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) bv[i] = 0.0f;
    if (a.bias == nullptr) return;
    if (o + N <= a.Cout && aligned16_dev(a.bias)) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const f32x4 q = *(const f32x4*)(a.bias + o + 4 * i);
            bv[4 * i] = q.x; bv[4 * i + 1] = q.y; bv[4 * i + 2] = q.z; bv[4 * i + 3] = q.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i)
            if (o + i < a.Cout) bv[i] = a.bias[o + i];
    }
}

template <typename T>
__device__ __forceinline__ void emit_run(const ConvArgs& a, bool to_y, bool vec_ok, long t, long pix, int o,
                                         float (&v)[Vec16<T>::N], const ActParams<Vec16<T>::N>& ap,
                                         bool early = false, uint4 early_tiles = make_uint4(0, 0, 0, 0),
                                         uint4 early_full = make_uint4(0, 0, 0, 0))
{
    constexpr int N = Vec16<T>::N;
    T* __restrict__ out = (T*)a.out;
    if (vec_ok && o + N <= a.Cout) {
        uint4 r;
        if (to_y && (a.res_tiles || a.res_full)) {
            float q[N];
            if (a.res_tiles) {
                uint4 rt = early_tiles;
                if (!early) rt = *(const uint4*)((const T*)a.res_tiles + t);
                unpack<T>(rt, q);
#pragma unroll
                for (int i = 0; i < N; ++i) v[i] += q[i];
            }
            if (a.res_full) {
                uint4 rf = early_full;
                if (!early) rf = *(const uint4*)((const T*)a.res_full + pix * a.res_ld + o);
                unpack<T>(rf, q);
#pragma unroll
                for (int i = 0; i < N; ++i) v[i] += q[i];
            }
        }
        r = pack<T>(v);
        if (to_y) {
            *(uint4*)((T*)a.y + pix * a.y_ld + o) = r;
            // the next layers' normalisation and nonlinearity, applied here once instead of by every
            // workgroup that later gathers this pixel (from the stored, rounded value)
#pragma unroll
            for (int j = 0; j < SIGE_MAX_ACT_OUTS; ++j) {
                if (j >= a.n_ao) break;
                float f[N];
                unpack<T>(r, f);
                scale_shift_act<N>(f, ap.sc[j], ap.sh[j], a.ao[j].act);
                *(uint4*)((T*)a.ao[j].y + pix * a.ao[j].ld + o) = pack<T>(f);
            }
        } else {
            *(uint4*)(out + t) = r;
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if (o + i >= a.Cout) break;
            float f = v[i];
            if (to_y) {
                if (a.res_tiles) f += to_f32(((const T*)a.res_tiles)[t + i]);
                if (a.res_full) f += to_f32(((const T*)a.res_full)[pix * a.res_ld + o + i]);
            }
            const T r = from_f32<T>(f);
            if (to_y) {
                ((T*)a.y)[pix * a.y_ld + o + i] = r;
            } else {
                out[t + i] = r;
            }
        }
    }
}

// One run of a gated-GELU output: v the N values, gt their gates (bias included in both), o the
// convolution channel of v[0] (o % 16 < 8): out[row][(o / 16) * 8 + o % 16 + i] = v[i] * gelu(gt[i]),
// gelu(g) = g/2 * (1 + erf(g / sqrt 2)), from the fp32 sums: the layer's one stored tensor is this
// product, rounded once.
template <typename T>
__device__ __forceinline__ void emit_glu(const ConvArgs& a, long row, int o, float (&v)[Vec16<T>::N],
                                         const float (&gt)[Vec16<T>::N])
{
    constexpr int N = Vec16<T>::N;
    const int Cg = a.Cout / 2, oo = (o >> 4) * 8 + (o & 15);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] *= 0.5f * gt[i] * (1.0f + erff(gt[i] * 0.70710678118654752f));
    T* dst = (T*)a.out + row * Cg + oo;
    if (Cg % N == 0 && aligned16_dev(a.out)) {
        *(uint4*)dst = pack<T>(v);
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) dst[i] = from_f32<T>(v[i]);
    }
}

// Whether the 16-byte paths of emit_run may be taken for this call.
template <typename T>
__device__ __forceinline__ bool emit_vec_ok(const ConvArgs& a)
{
    constexpr int N = Vec16<T>::N;
    return (a.Cout % N == 0) && aligned16_dev(a.out) &&
           (a.y == nullptr ||
            (a.y_ld % N == 0 && aligned16_dev(a.y) && (!a.res_tiles || aligned16_dev(a.res_tiles)) &&
             (!a.res_full || (a.res_ld % N == 0 && aligned16_dev(a.res_full)))));
}

// Largest divisor of the number of steps that does not exceed the limit.
constexpr int ring_depth(int steps, int limit)
{
    int d = 1;
    for (int i = 1; i <= limit && i <= steps; ++i)
        if (steps % i == 0) d = i;
    return d;
}

constexpr int MAX_G = 256;   // most blocks one workgroup can hold (1x1 blocks in a 256-row patch)

// TM x TN: 32x32 MFMA tiles per wave; WM x WN x WK = 4 (or 8) waves over M, N and K (waves that
// split K take different channel ranges of every tap and are summed through LDS at the end); KC =
// K steps per staged channel chunk; KK = k*k when it is 9 or 1 (the steps of a chunk are then
// unrolled), 0 for any other kernel size.  Two waves per SIMD are enforced: with fewer the MFMA
// phase has nothing to overlap its LDS and L2 latencies with.
// (The body is a device function so that two calls can share one launch, see conv_pair_kernel;
// bx, by, bz are the workgroup's coordinates inside its own call's grid.)
template <typename T, int TM, int TN, int WM, int WN, int WK, int KC, int KK, bool MARKED = false>
__device__ __forceinline__ void conv_body(const ConvArgs& a, const int bx, const int by, const int bz)
{
    constexpr int NT = 64 * WM * WN * WK;                     // threads per workgroup
    static_assert(NT == 256 || NT == 512, "four or eight waves per workgroup");
    static_assert(KC % WK == 0, "waves that split K take whole K steps");
    constexpr int KS = Mma<T>::KSTEP;
    constexpr int S = (int)sizeof(T);
    constexpr int KW = KC / WK;                               // K steps per wave and tap
    extern __shared__ uint4 lds4[];
    char* lds = reinterpret_cast<char*>(lds4);
    // the arguments, fetched in two goes instead of group by group before each first use
    asm volatile("" ::"s"(a.indices), "s"(a.count), "s"(a.max_blocks), "s"(a.n_host), "s"(a.G), "s"(a.bands),
                 "s"(a.rows), "s"(a.bh), "s"(a.bw), "s"(a.stride), "s"(a.trows), "s"(a.tw), "s"(a.th), "s"(a.ps),
                 "s"(a.k), "s"(a.Cin), "s"(a.Cout), "s"(a.w), "s"(a.bias), "s"(a.partial), "s"(a.ksplit),
                 "s"(a.x), "s"(a.tiles), "s"(a.scale), "s"(a.shift), "s"(a.act), "s"(a.x_ld), "s"(a.up),
                 "s"(a.pad), "s"(a.Hin));
    asm volatile("" ::"s"(a.Win), "s"(a.y), "s"(a.y_ld), "s"(a.out), "s"(a.res_tiles), "s"(a.res_full),
                 "s"(a.res_ld), "s"(a.Hout), "s"(a.Wout), "s"(a.partial_stride), "s"(a.n_ao), "s"(a.ao[0].y),
                 "s"(a.ao[0].scale), "s"(a.ao[0].shift), "s"(a.ao[0].ld), "s"(a.ao[0].act), "s"(a.ao[1].y),
                 "s"(a.ao[1].scale), "s"(a.ao[1].shift), "s"(a.ao[1].ld), "s"(a.ao[1].act));

    // Fused mode: the origins of this workgroup's blocks go to LDS once.  Their loads and the
    // load of the count are independent and are issued together (row n exists for n < max_blocks).
    __shared__ int org[2 * MAX_G];
    const int g0 = bz * a.G;
    int n_eff;
    if constexpr (MARKED) {
        // Marked mode: the ordered list is the row-major sequence of the set flags (Sec. 3.2, the block
        // reduction).  A lane takes four flags (one 32-bit word: the workspace is 16-byte aligned and
        // padded), the lanes before it are counted with ballots of the bits of its own count, the waves
        // before it through LDS.  The workgroup keeps the origins of its own G slots; the first one of
        // the call stores the whole list and the count.
        // The flags of this step are in the half that the marking pass used (it left the phase it
        // read in the second phase word; both halves are fetched together with it, one round trip).
        // Nobody touches the other half during this step, so the call's first workgroup clears it
        // and advances the first phase word: the next marking pass finds a clean half without any
        // workgroup having to wait for the others to finish reading this one.
        static_assert(NT == 256, "marked mode is built for the four-wave shape");
        __shared__ int wtot[4];
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
        const uint32_t* words = reinterpret_cast<const uint32_t*>(a.mk_flags);
        const int hw = a.mk_half >> 2;
        uint32_t w0 = 0u, w1 = 0u;
        if (4 * tid < a.mk_nb) { w0 = words[tid]; w1 = words[hw + tid]; }
        const uint32_t phase = words[2 * hw + 1];
        const uint32_t w = (phase & 1u) ? w1 : w0;
        const bool writer = bx == 0 && by == 0 && bz == 0;
        if (writer) {
            uint4* other = reinterpret_cast<uint4*>(a.mk_flags + ((phase & 1u) ? 0 : a.mk_half));
            for (int i = tid; i < (a.mk_half >> 4); i += NT) other[i] = make_uint4(0, 0, 0, 0);
            if (tid == 0) reinterpret_cast<uint32_t*>(a.mk_flags)[2 * hw] = phase + 1u;
        }
        int f[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = ((w >> (8 * j)) & 0xffu) != 0u && 4 * tid + j < a.mk_nb;
        const int c = f[0] + f[1] + f[2] + f[3];
        const unsigned long long b0 = __ballot(c & 1), b1 = __ballot(c & 2), b2 = __ballot(c & 4);
        const unsigned long long lt = (1ull << lane) - 1ull;
        const int pre = __popcll(b0 & lt) + 2 * __popcll(b1 & lt) + 4 * __popcll(b2 & lt);
        if (lane == 0) wtot[wave] = __popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2);
        __syncthreads();
        int off = 0, total = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = wtot[i];
            if (i < wave) off += t;
            total += t;
        }
        int slot = off + pre;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (f[j]) {
                const int blk = 4 * tid + j;
                int byy, bxx;
                divmod(blk, a.d_mk_nbx, byy, bxx);
                const int oy = byy * a.bh, ox = bxx * a.bw;
                if (slot >= g0 && slot < g0 + a.G) { org[2 * (slot - g0)] = oy; org[2 * (slot - g0) + 1] = ox; }
                if (writer && slot < a.max_blocks) { a.mk_indices[2 * slot] = oy; a.mk_indices[2 * slot + 1] = ox; }
                ++slot;
            }
        }
        if (writer && tid == 0) *a.mk_count = total;
        n_eff = min(total, a.max_blocks);
        __syncthreads();
        if (g0 >= n_eff) return;
    } else {
        int oy = 0, ox = 0;
        if (a.indices != nullptr && threadIdx.x < a.G) {
            const int n = min(g0 + (int)threadIdx.x, a.max_blocks - 1);
            oy = a.indices[2 * n];
            ox = a.indices[2 * n + 1];
        }
        n_eff = effective_blocks(a.count, a.max_blocks, a.n_host);
        asm volatile("" : "+v"(oy), "+v"(ox), "+v"(n_eff));
        if (g0 >= n_eff) return;
        if (a.indices != nullptr) {
            if (threadIdx.x < a.G) { org[2 * threadIdx.x] = oy; org[2 * threadIdx.x + 1] = ox; }
            __syncthreads();
        }
    }
    // (a compiler-made division is some forty dependent instructions, 0.15 us on the path of every workgroup)
    int split, band;
    divmod(by, a.d_bands, split, band);
    const int band_row0 = band * a.rows;                      // first output row of the band
    const int band_rows = min(a.rows, a.bh - band_row0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wmn = wave / WK;
    const int wm = wmn / WN, wn = wmn - wm * WN;
    const int half = lane >> 5, l32 = lane & 31;
    const int trow0 = band_row0 * a.stride;                   // first staged tile row

    // LDS byte offset of this lane's A row for each of its M tiles (clamped to a valid pixel)
    int a_base[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = (wm * TM + tm) * 32 + l32;
        int g, p, py, px;
        divmod(m, a.d_pb, g, p);
        divmod(p, a.d_bw, py, px);
        if (g >= a.G || py >= band_rows) { g = 0; py = 0; px = 0; }
        a_base[tm] = ((g * a.trows + py * a.stride) * a.tw + px * a.stride) * a.ps + half * 16 +
                     wk * KW * (KS * S);
    }
    const int nt0 = (bx * WN + wn) * TN;                      // first 32-wide Cout tile of this wave
    const int kk = a.k * a.k, kcs = a.Cin / KS;
    const int ntn_total = (a.Cout + 31) / 32;

    // The bias is fetched now and added when the accumulators leave the registers, so that its
    // load latency hides behind the whole K loop instead of delaying the first MFMA.
    // Shapes whose waves do not split K multiply with the operands swapped (weights as the first,
    // pixels as the second): a lane then owns ONE pixel of a 32 x 32 tile and registers 4g .. 4g+3 hold
    // its channels 8g + 4*half .. + 3, so the accumulators can leave straight from the registers in
    // 16-byte channel runs (no trip through LDS, no barrier).  Their bias is folded into the start value
    // of the accumulators; the other shapes add it when the waves' sums meet in LDS.
    constexpr bool SWAP = WK == 1;
    // The start values are only requested here (four-float vectors where the run is whole) and go into
    // the accumulators after the first chunk is staged: taken at once they would make every workgroup
    // wait for a round trip to memory before it has asked for its weights and its tile.
    f32x16 acc[TM][TN];
    f32x16 acc_init[TN];
    float bias_v[TN];
    const bool bias4 = aligned16_dev(a.bias);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int o = (nt0 + tn) * 32 + l32;
        bias_v[tn] = (!SWAP && a.bias && o < a.Cout && wk == 0 && a.partial == nullptr) ? a.bias[o] : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_init[tn][r] = 0.0f;
        if (SWAP && a.bias != nullptr && a.partial == nullptr) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ob = (nt0 + tn) * 32 + 8 * g + 4 * half;
                if (bias4 && ob + 4 <= a.Cout) {
                    const f32x4 q = *(const f32x4*)(a.bias + ob);
                    acc_init[tn][4 * g] = q.x; acc_init[tn][4 * g + 1] = q.y;
                    acc_init[tn][4 * g + 2] = q.z; acc_init[tn][4 * g + 3] = q.w;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc_init[tn][4 * g + i] = ob + i < a.Cout ? a.bias[ob + i] : 0.0f;
                }
            }
        }
    }
    auto start_accumulators = [&]() {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = acc_init[tn];
    };

    // weight fragment pointers of this wave's Cout tiles (at tap 0, this wave's first K step)
    const uint4* __restrict__ wp[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int nt = min(nt0 + tn, ntn_total - 1);
        wp[tn] = (const uint4*)a.w + ((long)nt * kk * kcs + wk * KW) * 64 + lane;
    }
    const char* __restrict__ tiles = (const char*)a.tiles;
    const int npix = a.G * a.trows * a.tw;
    constexpr int VPC = KC * KS * S / 16;                     // 16-byte vectors per staged pixel

    // Weight fragments run D steps ahead of the MFMAs in a register ring (a step = one K step of one
    // tap: TM x TN MFMAs).  The steps of one channel chunk are unrolled into straight-line code (KK =
    // k*k known at compile time), so every ring slot is a fixed register and the hardware's in-order
    // load counter lets the oldest slot be awaited while the younger loads stay in flight.  D divides
    // the steps of a chunk; a prefetch that would run past the last chunk re-reads the last chunk
    // instead of branching.  Small rings throughout: in the K-split shape, whose calls are latency
    // bound, fetching the whole chunk ahead (18 loads per wave) holds up the tile loads behind it by
    // more than it saves later (measured 7.5 vs 7.9 us on a 9-block call with 6 vs 18 slots).
    constexpr int STEPS = KK > 0 ? KK * KW : 1;
    constexpr int D = KK == 0 ? 1 : ring_depth(STEPS, TN == 1 ? 6 : 8);
    const int nch = a.Cin / (KC * KS);
    int ch0 = 0, ch1 = nch, rem_unused;                       // this workgroup's chunks
    if (a.ksplit > 1) {
        divmod(split * nch, a.d_ksplit, ch0, rem_unused);
        divmod((split + 1) * nch, a.d_ksplit, ch1, rem_unused);
    }
    const int ntaps = KK ? KK : kk;
    uint4 ring[D][TN];
    auto fetch = [&](uint4 (&slot)[TN], int chunk, int tp, int kc) {
        chunk = min(chunk, nch - 1);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) slot[tn] = wp[tn][((long)tp * kcs + chunk * KC + kc) * 64];
    };
    const bool fused = a.x != nullptr;
    const bool fuse_math = fused && (a.scale != nullptr || a.act != SIGE_ACT_NONE);
    // Staging of one channel chunk.  The staging threads are a multiple of VPC (the few left over when
    // VPC does not divide NT sit the staging out), so a thread keeps one 16-byte channel
    // group and walks over the pixels NT / VPC at a time without dividing.  Each batch of U vectors
    // is loaded before any of them is used (addresses are clamped into the source, so the loads are
    // unconditional and overlap; what lies outside becomes zero afterwards).
    constexpr int U = TM * TN >= 4 ? 6 : 8;                   // fewer where the accumulators leave fewer registers
    constexpr int PPI = NT / VPC;                             // pixels covered by one step of the walk
    constexpr int NTS = PPI * VPC;                            // threads that stage (all of them unless VPC is 40 or 80)
    const int sv = tid % VPC;
    int sq0 = tid < NTS ? tid / VPC : npix, sg0, sr0, sx0;    // first pixel of this thread: index, block, row, column
    int step_g, step_r, step_x;                               // PPI pixels further, in the same mixed radix
    {
        int rem;
        divmod(sq0, a.d_per, sg0, rem);
        divmod(rem, a.d_tw, sr0, sx0);
        divmod(PPI, a.d_per, step_g, rem);
        divmod(rem, a.d_tw, step_r, step_x);
    }
    const int Ws = a.Win >> a.up;
    const int rmax = a.th - 1 - trow0;                        // last staged row that exists in the tile
    // FUSED: gather from x instead of reading stored tiles; SINGLE: one block per workgroup, whose
    // origin is then fixed.  Both are decided once per call, outside the per-vector code.
    auto stage_as = [&](int chunk, auto fused_c, auto single_c) {
        constexpr bool FUSED = decltype(fused_c)::value, SINGLE = decltype(single_c)::value;
        constexpr int N = Vec16<T>::N;
        const int c0 = chunk * (KC * KS);
        if (chunk != ch0) __syncthreads();
        float sc[N], sh[N];
        if (FUSED && fuse_math) {
            const int cbase = c0 + sv * N;                     // a multiple of N: whole 16-byte vectors
#pragma unroll
            for (int i = 0; i < N; ++i) { sc[i] = 1.0f; sh[i] = 0.0f; }
            if (a.scale != nullptr) {
                if (aligned16_dev(a.scale) && aligned16_dev(a.shift)) {
#pragma unroll
                    for (int i = 0; i < N / 4; ++i) {
                        const f32x4 c = *(const f32x4*)(a.scale + cbase + 4 * i), h = *(const f32x4*)(a.shift + cbase + 4 * i);
                        sc[4 * i] = c.x; sc[4 * i + 1] = c.y; sc[4 * i + 2] = c.z; sc[4 * i + 3] = c.w;
                        sh[4 * i] = h.x; sh[4 * i + 1] = h.y; sh[4 * i + 2] = h.z; sh[4 * i + 3] = h.w;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < N; ++i) { sc[i] = a.scale[cbase + i]; sh[i] = a.shift[cbase + i]; }
                }
            }
        }
        // this thread's 16 bytes of pixel 0 of the source; pixels are then a 32-bit index away
        const char* const src0 = (FUSED ? (const char*)a.x : tiles) + (long)c0 * S + sv * 16;
        const int px_bytes = (FUSED ? a.x_ld : a.Cin) * S;
        int q = sq0, g = sg0, r = sr0, x = sx0;
        int gc = -1, oyb = 0, oxb = 0, tb = 0;                 // block the cached origin belongs to
        auto origin = [&](int gg) {
            gc = gg;
            if (FUSED) {
                const int gl = min(gg, a.G - 1);
                oyb = org[2 * gl] * a.stride - a.pad + trow0;
                oxb = org[2 * gl + 1] * a.stride - a.pad;
            } else {
                tb = (min(g0 + gg, n_eff - 1) * a.th + trow0) * a.tw;
            }
        };
        if (SINGLE) origin(0);
        while (q < npix) {
            uint4 val[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!SINGLE && g != gc) origin(g);
                ok[u] = q + u * PPI < npix && r <= rmax && (SINGLE || g0 + g < n_eff);
                const int rr = min(r, rmax);
                int pix;
                if (!FUSED) {
                    pix = tb + rr * a.tw + x;
                } else {
                    // the gather: input pixel of tile position (trow0 + r, x) of block g0 + g
                    const int iy = oyb + rr, ix = oxb + x;
                    ok[u] = ok[u] && iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win;
                    pix = (min(max(iy, 0), a.Hin - 1) >> a.up) * Ws + (min(max(ix, 0), a.Win - 1) >> a.up);
                }
                val[u] = *(const uint4*)(src0 + (long)pix * px_bytes);
                x += step_x;
                r += step_r;
                if (x >= a.tw) { x -= a.tw; ++r; }
                if (!SINGLE) {
                    g += step_g;
                    if (r >= a.trows) { r -= a.trows; ++g; }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (q + u * PPI >= npix) break;
                // computed for every vector, selected afterwards: no branch between the vectors of a
                // batch, so their chains interleave; padding and inactive rows stay literally zero
                uint4 w = val[u];
                if (FUSED && fuse_math) {
                    float f[N];
                    unpack<T>(w, f);
                    scale_shift_act<N>(f, sc, sh, a.act);
                    w = pack<T>(f);
                }
                if (!ok[u]) w = make_uint4(0, 0, 0, 0);
                *(uint4*)(lds + (q + u * PPI) * a.ps + sv * 16) = w;
            }
            q += U * PPI;
        }
        __syncthreads();
    };
    auto stage = [&](int chunk) {
        using yes = std::true_type;
        using no = std::false_type;
        if (fused) {
            if (a.G == 1) stage_as(chunk, yes{}, yes{});
            else stage_as(chunk, yes{}, no{});
        } else {
            if (a.G == 1) stage_as(chunk, no{}, yes{});
            else stage_as(chunk, no{}, no{});
        }
    };
    auto load_a = [&](uint4 (&af)[TM], int tp, int kc) {
        const int kdim = KK == 9 ? 3 : (KK == 1 ? 1 : a.k);      // known at compile time for the unrolled sizes
        const int ky = tp / kdim, kx = tp - ky * kdim;
        const int off = (ky * a.tw + kx) * a.ps + kc * (KS * S);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) af[tm] = *(const uint4*)(lds + a_base[tm] + off);
    };
    auto multiply = [&](const uint4 (&af)[TM], const uint4 (&b)[TN]) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                if constexpr (SWAP) Mma<T>::run(b[tn], af[tm], acc[tm][tn]);
                else Mma<T>::run(af[tm], b[tn], acc[tm][tn]);
            }
    };

    if constexpr (KK > 0) {
#pragma unroll
        for (int d = 0; d < D; ++d) fetch(ring[d], ch0, d / KW, d % KW);
        // (shapes with start values from memory stage the first chunk ahead of the loop, so that those values
        // are dead before the loop begins; the others keep the one staging site - their kernels start cold in a
        // network step and every kilobyte of code is fetched first)
        if constexpr (SWAP) stage(ch0);
        start_accumulators();
        for (int chunk = ch0; chunk < ch1; ++chunk) {
            if (!SWAP || chunk != ch0) stage(chunk);
            // A rows run AD steps ahead of their MFMAs: one step where a step holds four MFMAs or
            // more, two where it holds fewer and would not cover the LDS latency.  In the small shapes
            // a barrier after the loads keeps them in front of this step's MFMAs (the scheduler
            // otherwise issues them behind, and every step then waits for its own rows); the large
            // shape is faster with the scheduler left free inside a step.
            constexpr int AD = TM * TN >= 4 ? 1 : (STEPS > 2 ? 2 : 1);
            uint4 af[AD + 1][TM];
#pragma unroll
            for (int i = 0; i < AD; ++i) load_a(af[i], i / KW, i % KW);
#pragma unroll
            for (int st = 0; st < STEPS; ++st) {
                if (st + AD < STEPS) load_a(af[(st + AD) % (AD + 1)], (st + AD) / KW, (st + AD) % KW);
                if constexpr (TM * TN < 4) __builtin_amdgcn_sched_barrier(0);
                multiply(af[st % (AD + 1)], ring[st % D]);
                const int nx = (st + D) % STEPS;              // the step that takes over this slot
                fetch(ring[st % D], st + D < STEPS ? chunk : chunk + 1, nx / KW, nx % KW);
                // nothing moves across a step boundary: left alone, the scheduler sinks every prefetch
                // down to its first use to save registers and the ring collapses
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
        start_accumulators();
        for (int chunk = ch0; chunk < ch1; ++chunk) {
            stage(chunk);
#pragma nounroll
            for (int tp = 0; tp < ntaps; ++tp)
#pragma unroll
                for (int kc = 0; kc < KW; ++kc) {
                    uint4 af[TM];
                    fetch(ring[0], chunk, tp, kc);
                    load_a(af, tp, kc);
                    multiply(af, ring[0]);
                }
        }
    }

    // ---- epilogue.  Shapes with swapped operands send whole 16-byte channel runs straight from the
    // registers (a lane owns a pixel).  Otherwise - waves that split K, a gated GELU, partial sums of a K
    // split over workgroups, ragged channel counts - the accumulators go through LDS (the staged tile is
    // no longer needed) so that every thread then owns 8 consecutive output channels of one pixel.
    constexpr int N = Vec16<T>::N;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr int RS = BN + 4;                                // fp32 row stride: pad keeps 16-byte alignment
    float* red = reinterpret_cast<float*>(lds);               // [WK][BM][RS]
    const bool vec_ok = emit_vec_ok<T>(a);
    const bool to_y = a.y != nullptr;                    // scatter epilogue (block origins given)
    if constexpr (SWAP) {
        // Straight from the registers: whole 16-byte runs, no gated GELU, no K split over workgroups
        // (everything else takes the path through LDS below).
        if (vec_ok && !a.glu && a.partial == nullptr && a.direct) {
            constexpr int RL = N == 8 ? 2 : 4;            // runs of N channels this lane emits per 32 x 32 tile
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int m = (wm * TM + tm) * 32 + l32;
                int g, p, py, px;
                divmod(m, a.d_pb, g, p);
                divmod(p, a.d_bw, py, px);
                bool valid = g < a.G && py < band_rows && g0 + g < n_eff;
                long pix = 0;
                if (to_y && valid) {
                    const int oy = org[2 * g] + band_row0 + py, ox = org[2 * g + 1] + px;
                    valid = oy >= 0 && oy < a.Hout && ox >= 0 && ox < a.Wout;
                    pix = (long)oy * a.Wout + ox;
                }
                const long trow = (((long)(g0 + g) * a.bh + band_row0 + py) * a.bw + px) * a.Cout;
                const bool res = to_y && valid && (a.res_tiles != nullptr || a.res_full != nullptr);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    // the residual vectors of this tile's runs do not depend on the sums: fetched together first
                    uint4 et[RL], ef[RL];
#pragma unroll
                    for (int j = 0; j < RL; ++j) {
                        const int o = (nt0 + tn) * 32 + (N == 8 ? 16 * j + 8 * half : 8 * j + 4 * half);
                        et[j] = ef[j] = make_uint4(0, 0, 0, 0);
                        if (res && o < a.Cout) {
                            if (a.res_tiles) et[j] = *(const uint4*)((const T*)a.res_tiles + trow + o);
                            if (a.res_full) ef[j] = *(const uint4*)((const T*)a.res_full + pix * a.res_ld + o);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < RL; ++j) {
                        float v[N];
                        int o;
                        if constexpr (N == 8) {
                            // groups 2j (channels 16j .. 16j+7 split over the lane halves) and 2j+1: the lower
                            // half of the wave takes the first run and hands over its share of the second
                            o = (nt0 + tn) * 32 + 16 * j + 8 * half;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float first = acc[tm][tn][8 * j + i], second = acc[tm][tn][8 * j + 4 + i];
                                const float got = __shfl_xor(half ? first : second, 32);       // the partner's share of my run
                                v[i] = half ? got : first;
                                v[4 + i] = half ? second : got;
                            }
                        } else {
                            o = (nt0 + tn) * 32 + 8 * j + 4 * half;
#pragma unroll
                            for (int i = 0; i < 4; ++i) v[i] = acc[tm][tn][4 * j + i];
                        }
                        if (!valid || o >= a.Cout) continue;
                        ActParams<N> ap;
                        load_act_params<N>(a, o, ap);
                        emit_run<T>(a, to_y, true, trow + o, pix, o, v, ap, true, et[j], ef[j]);
                    }
                }
            }
            return;
        }
    }
    {
        __syncthreads();
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // (swapped operands: the lane is the pixel and the registers are the channels)
                    const int rr = 8 * (r >> 2) + 4 * half + (r & 3);
                    const int m = (wm * TM + tm) * 32 + (SWAP ? l32 : rr);
                    const int nn = (wn * TN + tn) * 32 + (SWAP ? rr : l32);
                    red[(wk * BM + m) * RS + nn] = acc[tm][tn][r] + bias_v[tn];
                }
        __syncthreads();
        for (int e = tid; e < BM * (BN / N); e += NT) {
            const int m = e / (BN / N), nn = (e - m * (BN / N)) * N;   // row of the workgroup's patch
            const int o = bx * BN + nn;
            int g, p, py, px;
            divmod(m, a.d_pb, g, p);
            divmod(p, a.d_bw, py, px);
            if (g >= a.G || py >= band_rows || g0 + g >= n_eff || o >= a.Cout) continue;
            if (a.glu) {          // value runs finish themselves and their gates, gate runs have nothing to do
                if ((o & 15) >= 8) continue;
                float v[N], gt[N];
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    v[i] = gt[i] = 0.0f;
#pragma unroll
                    for (int w = 0; w < WK; ++w) {
                        v[i] += red[(w * BM + m) * RS + nn + i];
                        gt[i] += red[(w * BM + m) * RS + nn + 8 + i];
                    }
                }
                emit_glu<T>(a, ((long)(g0 + g) * a.bh + band_row0 + py) * a.bw + px, o, v, gt);
                continue;
            }
            ActParams<N> ap;
            if (vec_ok && o + N <= a.Cout) load_act_params<N>(a, o, ap);
            float v[N];
#pragma unroll
            for (int i = 0; i < N; ++i) {
                v[i] = 0.0f;
#pragma unroll
                for (int w = 0; w < WK; ++w) v[i] += red[(w * BM + m) * RS + nn + i];
            }
            const long t = (((long)(g0 + g) * a.bh + band_row0 + py) * a.bw + px) * a.Cout + o;
            if (a.partial != nullptr) {      // this workgroup's share of K, unrounded, for the reduction kernel
                float* __restrict__ dst = a.partial + split * a.partial_stride + t;
                if ((a.Cout & 3) == 0 && o + N <= a.Cout) {
#pragma unroll
                    for (int i = 0; i < N; i += 4) *(float4*)(dst + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
                } else {
#pragma unroll
                    for (int i = 0; i < N; ++i)
                        if (o + i < a.Cout) dst[i] = v[i];
                }
                continue;
            }
            long pix = 0;
            if (to_y) {
                const int oy = org[2 * g] + band_row0 + py, ox = org[2 * g + 1] + px;
                if (oy < 0 || oy >= a.Hout || ox < 0 || ox >= a.Wout) continue;
                pix = (long)oy * a.Wout + ox;
            }
            emit_run<T>(a, to_y, vec_ok, t, pix, o, v, ap);
        }
    }
}

template <typename T, int TM, int TN, int WM, int WN, int WK, int KC, int KK>
__global__ __launch_bounds__(64 * WM * WN * WK, (WM * WN * WK > 4 ? 1 : 2)) void conv_kernel(ConvArgs a)
{
    if constexpr (WK == 1 && TM * TN >= 4) {
        // A workgroup's life is staging, then MFMA, then the epilogue; the two workgroups that share a
        // compute unit start together and would go through these phases in step for the whole launch
        // (memory, matrix pipes and memory again taking turns).  Half of the first round starts late,
        // which puts the co-resident workgroups out of phase; later rounds inherit the offset.
        if (a.stagger > 0) {
            const unsigned id = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
            if (id < 512u && (id & 1u))
                for (int i = 0; i < a.stagger; ++i) __builtin_amdgcn_s_sleep(127);
        }
    }
    conv_body<T, TM, TN, WM, WN, WK, KC, KK>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Two independent calls in ONE launch: a 3x3 convolution and a 1x1 convolution that both take the
// 64 x 32 shape whose four waves split K (few active blocks: a ResBlock's convolution and its
// shortcut, which read the same tensor).
// MARKED: the launch follows the marking pass directly, without the compaction pass in between (on
// this part a dependent launch costs more than the compaction's work): every workgroup derives its
// blocks from the flags (see conv_body).
template <typename T, int KC, bool MARKED>
__global__ __launch_bounds__(256, 2) void conv_pair_kernel(ConvArgs a, ConvArgs b, int wgs_a, FastDiv xa, FastDiv ya,
                                                           int ta, FastDiv xb, FastDiv yb, int tb)
{
    // A one-dimensional grid: the first call's workgroups, then the second's.  Consecutive workgroups
    // go to the eight XCDs in turn and each XCD has its own L2, so the workgroups that read the same
    // input tile (one per 32-wide slab of output channels) are numbered eight apart: they land on one
    // XCD and the tile leaves HBM once instead of once per slab.  (ta, tb: tiles = bands * groups.)
    int id = blockIdx.x;
    const bool first = id < wgs_a;
    if (!first) id -= wgs_a;
    const FastDiv nx = first ? xa : xb, ny = first ? ya : yb;
    const int nt = first ? ta : tb;
    int jt, bx, bz, by;
    divmod(id >> 3, nx, jt, bx);
    const int tile = jt * 8 + (id & 7);
    if (tile >= nt) return;
    divmod(tile, ny, bz, by);
    if (first) conv_body<T, 2, 1, 1, 1, 4, KC, 9, MARKED>(a, bx, by, bz);
    else conv_body<T, 2, 1, 1, 1, 4, KC, 1, MARKED>(b, bx, by, bz);
}

// v += the ksplit shares of one run of N channels, B of them in flight at a time (each batch is a
// round trip to memory), added in the order of the split index.
template <int B, int N>
__device__ __forceinline__ void add_shares(const float* __restrict__ partial, long stride, int ksplit, long t,
                                           float (&v)[N])
{
    for (int s0 = 0; s0 < ksplit; s0 += B) {
        f32x4 q[B][N / 4];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const float* __restrict__ src = partial + min(s0 + j, ksplit - 1) * stride + t;
#pragma unroll
            for (int i = 0; i < N / 4; ++i) q[j][i] = *(const f32x4*)(src + 4 * i);
        }
#pragma unroll
        for (int j = 0; j < B; ++j) {
            if (s0 + j < ksplit) {
#pragma unroll
                for (int i = 0; i < N / 4; ++i) {
                    v[4 * i] += q[j][i].x; v[4 * i + 1] += q[j][i].y;
                    v[4 * i + 2] += q[j][i].z; v[4 * i + 3] += q[j][i].w;
                }
            }
        }
    }
}

// Second kernel of a K-split call: adds the workgroups' shares in a fixed order, then the bias, and
// finishes every run of output channels exactly as the unsplit epilogue does.
template <typename T>
__global__ __launch_bounds__(256) void conv_reduce_kernel(ConvArgs a, long n_runs)
{
    constexpr int N = Vec16<T>::N;
    // every argument this kernel reads, fetched in one go
    asm volatile("" ::"s"(a.Cout), "s"(a.bh), "s"(a.bw), "s"(a.y), "s"(a.count), "s"(a.max_blocks), "s"(a.n_host),
                 "s"(a.indices), "s"(a.Hout), "s"(a.Wout), "s"(a.y_ld), "s"(a.res_tiles), "s"(a.res_full),
                 "s"(a.res_ld), "s"(a.bias), "s"(a.partial), "s"(a.partial_stride), "s"(a.ksplit), "s"(a.out),
                 "s"(a.n_ao), "s"(a.ao[0].y), "s"(a.ao[0].scale), "s"(a.ao[0].shift), "s"(a.ao[0].ld),
                 "s"(a.ao[0].act), "s"(a.ao[1].y), "s"(a.ao[1].scale), "s"(a.ao[1].shift), "s"(a.ao[1].ld),
                 "s"(a.ao[1].act));
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= n_runs) return;
    int row, run, n, p, py, px;                          // e < 2^31 (checked at the launch)
    divmod((int)e, a.d_runs, row, run);
    const int o = run * N;
    divmod(row, a.d_pbfull, n, p);
    divmod(p, a.d_bw, py, px);
    const bool to_y = a.y != nullptr;                    // scatter epilogue (block origins given)
    int y0 = 0, x0 = 0, n_eff;
    if (to_y) n_eff = blocks_and_origin(a.count, a.max_blocks, a.n_host, a.indices, n, y0, x0);
    else n_eff = effective_blocks(a.count, a.max_blocks, a.n_host);
    if (n >= n_eff) return;
    const long t = (long)row * a.Cout + o;
    long pix = 0;
    if (to_y) {
        const int oy = y0 + py, ox = x0 + px;
        if (oy < 0 || oy >= a.Hout || ox < 0 || ox >= a.Wout) return;
        pix = (long)oy * a.Wout + ox;
    }
    // the residual vectors do not depend on the sums: fetch them first so that they travel together
    // with the shares
    const bool vec_ok = emit_vec_ok<T>(a);
    const bool early_ok = to_y && vec_ok && o + N <= a.Cout;
    uint4 early_t = make_uint4(0, 0, 0, 0), early_f = make_uint4(0, 0, 0, 0);
    ActParams<N> ap;
    if (early_ok) {
        if (a.res_tiles) early_t = *(const uint4*)((const T*)a.res_tiles + t);
        if (a.res_full) early_f = *(const uint4*)((const T*)a.res_full + pix * a.res_ld + o);
        load_act_params<N>(a, o, ap);
    }
    float v[N], bv[N];
    const bool vec4 = (a.Cout & 3) == 0 && o + N <= a.Cout;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        v[i] = 0.0f;
    }
    load_bias<N>(a, o, bv);
    if (vec4) {
        if (a.ksplit <= 4) add_shares<4, N>(a.partial, a.partial_stride, a.ksplit, t, v);
        else if (a.ksplit <= 8) add_shares<8, N>(a.partial, a.partial_stride, a.ksplit, t, v);
        else add_shares<16, N>(a.partial, a.partial_stride, a.ksplit, t, v);
    } else {
        for (int s = 0; s < a.ksplit; ++s) {
            const float* __restrict__ src = a.partial + s * a.partial_stride + t;
#pragma unroll
            for (int i = 0; i < N; ++i)
                if (o + i < a.Cout) v[i] += src[i];
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += bv[i];
    emit_run<T>(a, to_y, vec_ok, t, pix, o, v, ap, early_ok, early_t, early_f);
}

// ---- 1x1 convolutions with few rows ------------------------------------------------------------
// A 1x1, stride-1 convolution on the stacked pixels of the active blocks is a matrix product with
// few rows (M = active pixels) and a long K; no input pixel is used by two taps, so a tile staged
// for the whole workgroup buys nothing.  One workgroup owns 64 rows x 32*TN output channels and its
// W waves split K: each streams its share of the rows' channels and of the packed weight into
// registers, P pairs of K steps ahead of the MFMAs, and the waves' sums meet in LDS, where they are
// added in wave order.  No second kernel, no workspace.
//
// Four neighbouring lanes fetch the 64 bytes that two K steps take from one row (a load instruction
// covers 16 rows, one request per row).  That is not the MFMA operand layout, so each pair of steps
// passes through a buffer in LDS that belongs to the wave alone: written as loaded, read back as
// operands, no workgroup barrier involved.
template <typename T, int W, int P, int TM, int TN>
__global__ __launch_bounds__(64 * W, W == 4 ? 2 : 1) void pointwise_kernel(ConvArgs a)
{
    constexpr int KS = Mma<T>::KSTEP, S = (int)sizeof(T), N = Vec16<T>::N;
    constexpr int BM = 32 * TM, BN = 32 * TN, RS = BN + 4;
    constexpr int NI = BM / 16;                               // load instructions per pair of K steps: 16 rows each
    constexpr int AROW = 80;                                  // bytes per row in the wave's buffer: 64 + pad
    constexpr int ABUF = BM * AROW;                           // one pair of K steps of the patch rows
    static_assert(2 * KS * S == 64, "two K steps of one row are 64 bytes");
    extern __shared__ uint4 lds4[];
    char* lds = reinterpret_cast<char*>(lds4);
    float* red = reinterpret_cast<float*>(lds4);              // [W][BM][RS], after the K loop
    // the arguments, fetched in two goes instead of group by group before each first use
    asm volatile("" ::"s"(a.w), "s"(a.Cin), "s"(a.Cout), "s"(a.bh), "s"(a.bw), "s"(a.x), "s"(a.tiles),
                 "s"(a.indices), "s"(a.count), "s"(a.max_blocks), "s"(a.n_host), "s"(a.Hin), "s"(a.Win),
                 "s"(a.x_ld), "s"(a.y), "s"(a.y_ld), "s"(a.out), "s"(a.res_tiles), "s"(a.res_full), "s"(a.res_ld),
                 "s"(a.bias), "s"(a.Hout), "s"(a.Wout), "s"(a.n_ao));
    asm volatile("" ::"s"(a.ao[0].y), "s"(a.ao[0].scale), "s"(a.ao[0].shift), "s"(a.ao[0].ld), "s"(a.ao[0].act),
                 "s"(a.ao[1].y), "s"(a.ao[1].scale), "s"(a.ao[1].shift), "s"(a.ao[1].ld), "s"(a.ao[1].act));
    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: the K loop is uniform
    const int pb = a.bh * a.bw;
    const int r0 = blockIdx.y * BM;
    const bool gathered = a.x != nullptr;                     // rows come from x at the blocks' pixels
    const bool have_org = a.indices != nullptr;               // needed by the gather and by the scatter epilogue
    const int kcs = a.Cin / KS, np = kcs / 2;                 // K steps, pairs of K steps
    const int q0 = wave * np / W, q1 = (wave + 1) * np / W;   // this wave's pairs
    const int ntn_total = (a.Cout + 31) / 32;

    // The weight fragments do not depend on the block list: their first loads go out before it is
    // read.  A fetch past the wave's share still happens, so that the loads in flight stay a fixed
    // number, but every lane then reads the same 16 bytes: one request instead of a kilobyte.
    const u32x4* const idle = (const u32x4*)a.w;
    const u32x4* __restrict__ wp[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
        wp[tn] = (const u32x4*)a.w + (long)min((int)blockIdx.x * TN + tn, ntn_total - 1) * kcs * 64 + lane;
    u32x4 ra[P][NI], rb[P][TN][2];
    auto fetch_b = [&](int st, int q) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const u32x4* src = q < q1 ? wp[tn] + (long)(2 * q) * 64 : idle;
            rb[st][tn][0] = src[0];
            rb[st][tn][1] = src[q < q1 ? 64 : 0];
        }
    };
#pragma unroll
    for (int st = 0; st < P; ++st) fetch_b(st, q0 + st);

    // rows this lane loads from: row 16*i + lane/4 of the patch, i < NI, clamped to rows that exist;
    // in fused mode the block origins are fetched together with the count (row n exists for
    // n < max_blocks)
    int oy[NI], ox[NI], rr[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        rr[i] = r0 + 16 * i + (lane >> 2);
        oy[i] = ox[i] = 0;
        if (have_org) {
            int n, rem_;
            divmod(rr[i], a.d_pbfull, n, rem_);
            n = min(n, a.max_blocks - 1);
            oy[i] = a.indices[2 * n];
            ox[i] = a.indices[2 * n + 1];
        }
    }
    int n_eff = effective_blocks(a.count, a.max_blocks, a.n_host);
#pragma unroll
    for (int i = 0; i < NI; ++i) asm volatile("" : "+v"(oy[i]), "+v"(ox[i]), "+v"(n_eff));
    const int rows = n_eff * pb;
    if (r0 >= rows) return;
    // the epilogue needs the origin of every row's block again: the first NI waves hold those of
    // rows 16*wave + lane/4 (the i = wave entry of what they just fetched)
    __shared__ int org[2 * BM];
    if (have_org && wave < NI && (lane & 3) == 0) {
        int yy = oy[0], xx = ox[0];
#pragma unroll
        for (int i = 1; i < NI; ++i)
            if (wave == i) { yy = oy[i]; xx = ox[i]; }
        org[2 * (16 * wave + (lane >> 2))] = yy;
        org[2 * (16 * wave + (lane >> 2)) + 1] = xx;
    }
    const char* __restrict__ rp[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int r = min(rr[i], rows - 1);
        long pixel = r;
        long ld = a.Cin;
        if (gathered) {
            int n, p, py, px;
            divmod(r, a.d_pbfull, n, p);
            divmod(p, a.d_bw, py, px);
            // the origin fetched above belongs to row rr; a clamped row reads the last block's
            const int y0 = r == rr[i] ? oy[i] : a.indices[2 * n];
            const int x0 = r == rr[i] ? ox[i] : a.indices[2 * n + 1];
            pixel = (long)min(y0 + py, a.Hin - 1) * a.Win + min(x0 + px, a.Win - 1);
            ld = a.x_ld;
        }
        rp[i] = (gathered ? (const char*)a.x : (const char*)a.tiles) + pixel * ld * S + (lane & 3) * 16;
    }
    auto fetch_a = [&](int st, int q) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
            ra[st][i] = *(q < q1 ? (const u32x4*)(rp[i] + (long)q * 64) : idle);
    };
#pragma unroll
    for (int st = 0; st < P; ++st) fetch_a(st, q0 + st);

    // What the epilogue needs for this thread's first run of output channels and does not depend on
    // the sums - bias and residuals - is fetched now and arrives during the K loop (the origin of the
    // run's row comes straight from the list: LDS holds it only later).
    const bool vec_ok = emit_vec_ok<T>(a);
    const bool to_y = a.y != nullptr;                    // scatter epilogue (block origins given)
    bool pre_ok = false;
    long pre_pix = 0;
    uint4 pre_t = make_uint4(0, 0, 0, 0), pre_f = make_uint4(0, 0, 0, 0);
    float pre_bv[N];
    {
        const int m = tid / (BN / N), nn = (tid - m * (BN / N)) * N;
        const int r = r0 + m, o = blockIdx.x * BN + nn;
#pragma unroll
        for (int i = 0; i < N; ++i) pre_bv[i] = 0.0f;
        if (tid < BM * (BN / N) && r < rows && o < a.Cout) {
            load_bias<N>(a, o, pre_bv);
            if (to_y && vec_ok && o + N <= a.Cout) {
                int n, p, py, px;
                divmod(r, a.d_pbfull, n, p);
                divmod(p, a.d_bw, py, px);
                const int yy = a.indices[2 * n] + py, xx = a.indices[2 * n + 1] + px;
                if (yy >= 0 && yy < a.Hout && xx >= 0 && xx < a.Wout) {
                    pre_ok = true;
                    pre_pix = (long)yy * a.Wout + xx;
                    if (a.res_tiles) pre_t = *(const uint4*)((const T*)a.res_tiles + (long)r * a.Cout + o);
                    if (a.res_full) pre_f = *(const uint4*)((const T*)a.res_full + pre_pix * a.res_ld + o);
                }
            }
        }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.0f;

    char* const abuf = lds + wave * (2 * ABUF);               // two buffers, used in turn
    const int a_wr = (lane >> 2) * AROW + (lane & 3) * 16;    // + 16 * i rows
    const int a_rd = l32 * AROW + half * 16;                  // + 32 * tm rows, + 32 bytes per step
    for (int q = q0; q < q1; q += P) {
#pragma unroll
        for (int st = 0; st < P; ++st) {
            {
                // no branch in the loop body: a stage past the wave's share multiplies zero rows, and the
                // number of loads in flight at every wait is known at compile time
                const bool live = q + st < q1;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                char* const buf = abuf + (st & 1) * ABUF;
#pragma unroll
                for (int i = 0; i < NI; ++i) *(u32x4*)(buf + 16 * i * AROW + a_wr) = live ? ra[st][i] : zero;
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const uint4 f0 = *(const uint4*)(buf + 32 * tm * AROW + a_rd);
                    const uint4 f1 = *(const uint4*)(buf + 32 * tm * AROW + a_rd + 32);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const u32x4 b0 = rb[st][tn][0], b1 = rb[st][tn][1];
                        Mma<T>::run(f0, make_uint4(b0.x, b0.y, b0.z, b0.w), acc[tm][tn]);
                        Mma<T>::run(f1, make_uint4(b1.x, b1.y, b1.z, b1.w), acc[tm][tn]);
                    }
                }
            }
            fetch_b(st, q + st + P);
            fetch_a(st, q + st + P);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // the waves' sums meet in LDS (the operand buffers are done with) and are added in wave order
    __syncthreads();
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = tm * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                red[(wave * BM + m) * RS + tn * 32 + l32] = acc[tm][tn][r];
            }
    __syncthreads();
    for (int e = tid; e < BM * (BN / N); e += 64 * W) {
        const int m = e / (BN / N), nn = (e - m * (BN / N)) * N;
        const int r = r0 + m, o = blockIdx.x * BN + nn;
        if (r >= rows || o >= a.Cout) continue;
        if (a.glu) {              // value runs finish themselves and their gates, gate runs have nothing to do
            if ((o & 15) >= 8) continue;
            float v[N], gt[N];
#pragma unroll
            for (int i = 0; i < N; ++i) { v[i] = 0.0f; gt[i] = 0.0f; }
            if (a.bias != nullptr) {      // whole runs: the channel count is a multiple of 16 here
                load_f32_run<N>(a.bias, o, v);
                load_f32_run<N>(a.bias, o + 8, gt);
            }
#pragma unroll
            for (int w = 0; w < W; ++w)
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    v[i] += red[(w * BM + m) * RS + nn + i];
                    gt[i] += red[(w * BM + m) * RS + nn + 8 + i];
                }
            emit_glu<T>(a, r, o, v, gt);
            continue;
        }
        const long t = (long)r * a.Cout + o;
        long pix = 0;
        if (to_y) {
            int n, p, py, px;
            divmod(r, a.d_pbfull, n, p);
            divmod(p, a.d_bw, py, px);
            const int yy = org[2 * m] + py, xx = org[2 * m + 1] + px;
            if (yy < 0 || yy >= a.Hout || xx < 0 || xx >= a.Wout) continue;
            pix = (long)yy * a.Wout + xx;
        }
        // bias and residuals do not depend on the sums: the first pass has them from the top of the
        // kernel, later passes fetch them before the sums are read
        const bool first = e == tid;
        const bool early_ok = to_y && vec_ok && o + N <= a.Cout;
        uint4 early_t = pre_t, early_f = pre_f;
        ActParams<N> ap;
        float v[N], bv[N];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            v[i] = 0.0f;
            bv[i] = pre_bv[i];
        }
        if (early_ok) {
            load_act_params<N>(a, o, ap);
            if (!(first && pre_ok)) {
                if (a.res_tiles) early_t = *(const uint4*)((const T*)a.res_tiles + t);
                if (a.res_full) early_f = *(const uint4*)((const T*)a.res_full + pix * a.res_ld + o);
            }
        }
        if (!first) {
#pragma unroll
            for (int i = 0; i < N; ++i) bv[i] = 0.0f;
            load_bias<N>(a, o, bv);
        }
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const float4* src = (const float4*)(red + (w * BM + m) * RS + nn);
#pragma unroll
            for (int i = 0; i < N / 4; ++i) {
                const float4 q = src[i];
                v[4 * i] += q.x; v[4 * i + 1] += q.y; v[4 * i + 2] += q.z; v[4 * i + 3] += q.w;
            }
        }
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += bv[i];
        emit_run<T>(a, to_y, vec_ok, t, pix, o, v, ap, early_ok, early_t, early_f);
    }
}

struct ConvPlan {
    int cfg;  // index into kCfg
    int kc;   // K steps per staged channel chunk: 8, 4 or 1; 16 to 40 in the shapes that stage the whole of Cin
    int G, rows, trows, Cc, ps, bands, slabs, groups;
    int ksplit;   // workgroups that share one output patch along K (1 = no split)
    size_t lds;
};

// M x N per workgroup and whether the four waves split K
struct CfgShape { int M, N, WK; };
constexpr int kNumCfg = 4;    // shapes that compete by score; the last two are chosen by a rule of their own
static const CfgShape kCfg[kNumCfg + 2] = {{128, 128, 1}, {128, 64, 1}, {64, 64, 1}, {64, 32, 4}, {64, 32, 8}, {32, 32, 8}};

template <typename T, int TM, int TN, int WM, int WN, int WK, int KC, int KK>
int launch_cfg(const ConvArgs& a, const ConvPlan& p, hipStream_t st)
{
    auto kern = conv_kernel<T, TM, TN, WM, WN, WK, KC, KK>;
    if (p.lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)p.lds);
        SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "sige_conv: cannot reserve %zu bytes of LDS: %s", p.lds,
                     hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, dim3(p.slabs, p.bands * p.ksplit, p.groups), dim3(64 * WM * WN * WK), p.lds, st, a);
    SIGE_LAUNCH_CHECK("sige_conv");
    return SIGE_OK;
}

template <typename T, int KC, int KK>
int launch_kc(const ConvArgs& a, const ConvPlan& p, hipStream_t st)
{
    switch (p.cfg) {
    case 0:
        if constexpr (KC <= 8) return launch_cfg<T, 2, 2, 2, 2, 1, KC, KK>(a, p, st);
        break;
    case 1:
        if constexpr (KC <= 8) return launch_cfg<T, 2, 1, 2, 2, 1, KC, KK>(a, p, st);
        break;
    case 2:
        if constexpr (KC <= 8) return launch_cfg<T, 1, 1, 2, 2, 1, KC, KK>(a, p, st);
        break;
    case 3:
        if constexpr (KC % 4 == 0 && (KC <= 8 || (KC == 20 && KK == 9))) return launch_cfg<T, 2, 1, 1, 1, 4, KC, KK>(a, p, st);
        break;
    case 4:
        if constexpr (KC % 8 == 0 && KC >= 16 && KK == 9) return launch_cfg<T, 2, 1, 1, 1, 8, KC, KK>(a, p, st);
        break;
    default:
        if constexpr (KC % 8 == 0 && KC >= 16 && KK == 9) return launch_cfg<T, 1, 1, 1, 1, 8, KC, KK>(a, p, st);
        break;
    }
    return fail(SIGE_ERR_UNSUPPORTED, "sige_conv: internal: shape %d without a matching chunk %d", p.cfg, KC);
}

template <typename T, int KK>
int launch_kk(const ConvArgs& a, const ConvPlan& p, hipStream_t st)
{
    switch (p.kc) {
    case 40: return launch_kc<T, 40, KK>(a, p, st);
    case 32: return launch_kc<T, 32, KK>(a, p, st);
    case 20: return launch_kc<T, 20, KK>(a, p, st);
    case 16: return launch_kc<T, 16, KK>(a, p, st);
    case 8: return launch_kc<T, 8, KK>(a, p, st);
    case 4: return launch_kc<T, 4, KK>(a, p, st);
    case 3: return launch_kc<T, 3, KK>(a, p, st);
    default: return launch_kc<T, 1, KK>(a, p, st);
    }
}

template <typename T>
int launch_conv(const ConvArgs& a, const ConvPlan& p, hipStream_t st)
{
    switch (a.k) {
    case 3: return launch_kk<T, 9>(a, p, st);
    case 1: return launch_kk<T, 1>(a, p, st);
    default: return launch_cfg<T, 1, 1, 2, 2, 1, 1, 0>(a, p, st);   // other kernel sizes: one plain shape
    }
}


template <typename T, int W, int P, int TM, int TN>
int launch_pointwise_as(const ConvArgs& a, int nl, hipStream_t st)
{
    auto kern = pointwise_kernel<T, W, P, TM, TN>;
    constexpr int BM = 32 * TM;
    const size_t lds = std::max((size_t)W * BM * (32 * TN + 4) * sizeof(float), (size_t)W * 2 * BM * 80);
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "sige_conv: cannot reserve %zu bytes of LDS: %s", lds,
                 hipGetErrorString(e));
    const int mt = (int)(((long)nl * a.bh * a.bw + BM - 1) / BM);
    hipLaunchKernelGGL(kern, dim3((a.Cout + 32 * TN - 1) / (32 * TN), mt), dim3(64 * W), lds, st, a);
    SIGE_LAUNCH_CHECK("sige_conv");
    return SIGE_OK;
}

template <typename T>
int launch_pointwise(const ConvArgs& a, int nl, int tiles, hipStream_t st)
{
    if (tiles == 3) return launch_pointwise_as<T, 8, 6, 1, 1>(a, nl, st);
    if (tiles == 2) {
        // more 64 x 64 patches than compute units: four waves per workgroup, so that two workgroups
        // share a compute unit and all of them run at once instead of in two rounds
        const long mt = ((long)nl * a.bh * a.bw + 63) / 64, nt2 = (a.Cout + 63) / 64;
        const int w4 = knob(SIGE_KNOB_CONV_POINTWISE_W4);      // 0 = never, 1 = always
        const bool four = w4 >= 0 ? w4 != 0 : mt * nt2 > 256;
        return four ? launch_pointwise_as<T, 4, 3, 2, 2>(a, nl, st) : launch_pointwise_as<T, 8, 3, 2, 2>(a, nl, st);
    }
    return launch_pointwise_as<T, 8, 4, 2, 1>(a, nl, st);
}

template <typename T>
int launch_reduce(const ConvArgs& a, int nl, hipStream_t st)
{
    const long n_runs = (long)nl * a.bh * a.bw * ((a.Cout + Vec16<T>::N - 1) / Vec16<T>::N);
    const long blocks = (n_runs + 255) / 256;
    SIGE_REQUIRE(n_runs < (1L << 31), SIGE_ERR_UNSUPPORTED, "sige_conv: too many output elements for the K-split reduction");
    hipLaunchKernelGGL((conv_reduce_kernel<T>), dim3((int)blocks), dim3(256), 0, st, a, n_runs);
    SIGE_LAUNCH_CHECK("sige_conv(reduce)");
    return SIGE_OK;
}

template <typename T>
int launch_pair(const ConvArgs& a, const ConvPlan& pa, const ConvArgs& b, const ConvPlan& pb, bool marked,
                hipStream_t st)
{
    const size_t lds = std::max(pa.lds, pb.lds);
    // tiles in groups of eight (one per XCD), every group times the slabs
    const int ta = pa.bands * pa.groups, tb = pb.bands * pb.groups;
    const int wgs_a = (ta + 7) / 8 * 8 * pa.slabs, wgs_b = (tb + 7) / 8 * 8 * pb.slabs;
    const dim3 grid(wgs_a + wgs_b);
    auto launch = [&](auto kern) {
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "sige_fused_conv_pair: cannot reserve %zu bytes of LDS: %s", lds,
                         hipGetErrorString(e));
        }
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, a, b, wgs_a, fast_div(pa.slabs), fast_div(pa.bands), ta,
                           fast_div(pb.slabs), fast_div(pb.bands), tb);
        SIGE_LAUNCH_CHECK("sige_fused_conv_pair");
        return (int)SIGE_OK;
    };
    if (marked) return pa.kc == 8 ? launch(conv_pair_kernel<T, 8, true>) : launch(conv_pair_kernel<T, 4, true>);
    return pa.kc == 8 ? launch(conv_pair_kernel<T, 8, false>) : launch(conv_pair_kernel<T, 4, false>);
}

// Re-lays an OIHW weight into the fragment order the kernels read.
template <typename T>
int launch_pack(const void* w_oihw, int Cout, int Cin, int k, long n, void* packed, hipStream_t st)
{
    const long blocks = (n + 255) / 256;
    hipLaunchKernelGGL((pack_weight_kernel<T>), dim3((int)blocks), dim3(256), 0, st, (const T*)w_oihw, Cout, Cin, k, n, (T*)packed);
    SIGE_LAUNCH_CHECK("sige_pack_weight");
    return SIGE_OK;
}

// The launchers one translation unit per storage type instantiates.
#define SIGE_CONV_LAUNCHERS(KW, T)                                                                              \
    KW template int launch_conv<T>(const ConvArgs&, const ConvPlan&, hipStream_t);                              \
    KW template int launch_pointwise<T>(const ConvArgs&, int, int, hipStream_t);                                \
    KW template int launch_reduce<T>(const ConvArgs&, int, hipStream_t);                                        \
    KW template int launch_pair<T>(const ConvArgs&, const ConvPlan&, const ConvArgs&, const ConvPlan&, bool, \
                                   hipStream_t);                                                            \
    KW template int launch_pack<T>(const void*, int, int, int, long, void*, hipStream_t);

}  // namespace sige
