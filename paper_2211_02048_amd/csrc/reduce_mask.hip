// sige_reduce_mask: difference mask (Sec. 3.1 "Structured sparsity"), per-scale
// downsample + dilate and reduction to the ordered active-block list (Sec. 3.2
// "Tiling-based sparse convolution", Fig. "method").
//
// Kernel 1 streams both activations once (the only HBM-sized traffic here): each
// lane owns one 16-byte vector, the lanes of one pixel vote with a wave ballot and
// the first lanes of the wave store one mask byte per pixel.
// With a caller workspace the block test is turned around: instead of every block
// scanning its tile, every MARKED pixel sets the flag of the (few) blocks whose
// dilated tile contains it - done by the difference kernel itself, or by a vectorised
// scan of a ready mask - and one small workgroup compacts the flags into the row-major
// list with an ordered ballot/popcount prefix sum and clears them for the next call.
// The flag workspace has two halves and two phase words behind them.  The marking pass writes into
// the half that the first phase word selects and copies that word into the second; the compaction
// reads and clears the same half.  A consumer that builds the list itself (conv_pair_kernel in
// marked mode, which follows the marking pass without a compaction launch) cannot clear the half its
// workgroups are still reading: it clears the OTHER half and advances the first phase word instead,
// so that the next marking pass finds a clean half.  Each phase word is written only by a kernel
// none of whose workgroups reads it.
// Without a workspace a single workgroup tests every block against the pooled, dilated
// mask (flags in LDS) and compacts.
#include "common.h"

#include <mutex>
#include <type_traits>

namespace sige {

template <typename T>
__device__ __forceinline__ bool vec_differs(const uint4& o, const uint4& e, float tau)
{
    float fo[Vec16<T>::N], fe[Vec16<T>::N];
    unpack<T>(o, fo);
    unpack<T>(e, fe);
    bool any = false;
#pragma unroll
    for (int i = 0; i < Vec16<T>::N; ++i) any |= !(fabsf(fe[i] - fo[i]) <= tau);
    return any;
}

struct MarkArgs {
    uint8_t* flags;  // the flag workspace: two halves of `half` bytes (one byte per block of the grid, padded to
                     // 16; the half in use is all zero on entry), then the two phase words
    int half;
    int pool_log2;
    int oy, ox;      // dilate + tile - pad: a pixel at pooled position p touches the blocks b with b*s > p - o ...
    int hi;          // dilate + pad:        ... and b*s <= p + hi
    int sy, sx;      // block pitch in input pixels: block * stride
    int nby, nbx;
    int ly, lx;      // base-2 logarithms of sy and sx where they are powers of two, else -1
    FastDiv dsy, dsx;   // division by sy and sx
};

__device__ __forceinline__ int fdiv(int x, const FastDiv& f)
{
    int q, r;
    divmod(x, f, q, r);
    return q;
}

// The lists one call builds from the same pooled mask (one per layer geometry at that resolution).
constexpr int MAX_LISTS = 4;
template <int NL>
struct MarkSetN {
    int n;           // lists in use (<= NL); 0 = do not mark
    int Wm, lW;      // source pixels per row; its base-2 logarithm if it is a power of two, else -1
    FastDiv dWm;
    MarkArgs m[NL > 0 ? NL : 1];
};
typedef MarkSetN<MAX_LISTS> MarkSet;

__device__ __forceinline__ uint32_t phase_of(const uint8_t* flags, int half)
{
    return *reinterpret_cast<const uint32_t*>(flags + 2 * half);
}

// The first thread of a marking launch leaves the phase it marks in where consumers look for it.
template <int NL>
__device__ __forceinline__ void publish_phase(const MarkSetN<NL>& mk)
{
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        if (i >= mk.n) break;
        uint32_t* p = reinterpret_cast<uint32_t*>(mk.m[i].flags + 2 * mk.m[i].half);
        p[1] = p[0];
    }
}

// Sets the flag of every block whose input tile, grown by the dilation radius, contains the
// pooled position of the marked source pixel (py, px).  In input coordinates block b covers
// [b*s - pad - r, b*s - pad + tile + r); clipping to the image never excludes an in-image pixel.
// A wave that marks is the slowest wave of a kernel that lasts a few microseconds, and what it
// executes here is one dependent chain (measured: 1.6 us for two lists with general divisions): block
// pitches that are powers of two - the usual case - take shifts, the others divisors prepared on the
// host, and the usual one or two blocks per axis are stored without a loop.
__device__ __forceinline__ void mark_blocks(const MarkArgs& m, uint32_t phase, int py, int px)
{
    const int y = py >> m.pool_log2, x = px >> m.pool_log2;
    const int ylo = y - m.oy, xlo = x - m.ox, yhi = y + m.hi, xhi = x + m.hi;
    int by0, bx0, by1, bx1;
    // first block with b*s > lo (a floor division that is also right for negative lo), last with b*s <= hi
    if (m.ly >= 0) {
        by0 = (ylo >> m.ly) + 1;
        by1 = yhi >> m.ly;
    } else {
        by0 = (ylo >= 0 ? fdiv(ylo, m.dsy) : -fdiv(-ylo + m.sy - 1, m.dsy)) + 1;
        by1 = fdiv(yhi, m.dsy);
    }
    if (m.lx >= 0) {
        bx0 = (xlo >> m.lx) + 1;
        bx1 = xhi >> m.lx;
    } else {
        bx0 = (xlo >= 0 ? fdiv(xlo, m.dsx) : -fdiv(-xlo + m.sx - 1, m.dsx)) + 1;
        bx1 = fdiv(xhi, m.dsx);
    }
    by0 = max(by0, 0);
    bx0 = max(bx0, 0);
    by1 = min(by1, m.nby - 1);
    bx1 = min(bx1, m.nbx - 1);
    if (by1 < by0 || bx1 < bx0) return;
    // Plain stores (the race is benign: every writer stores 1).  Looking at the flag first would
    // save stores but puts a dependent global load on the path of every marking lane.
    uint8_t* flags = m.flags + (phase & 1u) * m.half;
    uint8_t* f = flags + by0 * m.nbx + bx0;
    if (by1 - by0 <= 1 && bx1 - bx0 <= 1) {
        f[0] = 1;
        if (bx1 > bx0) f[1] = 1;
        if (by1 > by0) {
            f[m.nbx] = 1;
            if (bx1 > bx0) f[m.nbx + 1] = 1;
        }
        return;
    }
    for (int by = by0; by <= by1; ++by)
        for (int bx = bx0; bx <= bx1; ++bx) flags[by * m.nbx + bx] = 1;
}

// Row and column of source pixel `pix` (rows of Wm pixels; a shift when Wm is a power of two).
template <int NL>
__device__ __forceinline__ void pixel_rc(const MarkSetN<NL>& mk, int pix, int& py, int& px)
{
    if (mk.lW >= 0) {
        py = pix >> mk.lW;
        px = pix & (mk.Wm - 1);
    } else {
        divmod(pix, mk.dWm, py, px);
    }
}

// All lists' phase words (one round trip; lists beyond mk.n read the first list's word and are not used).
template <int NL>
__device__ __forceinline__ void load_phases(const MarkSetN<NL>& mk, uint32_t (&ph)[NL > 0 ? NL : 1])
{
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const bool used = i < mk.n;
        // (the address goes through a vector register that the compiler cannot see into: knowing it uniform,
        // it would move the word into a scalar register at once and wait for it in front of everything else)
        unsigned long long pv = reinterpret_cast<unsigned long long>((used ? mk.m[i].flags : mk.m[0].flags) +
                                                                     2 * (used ? mk.m[i].half : mk.m[0].half));
        asm volatile("" : "+v"(pv));
        // (as a pointer into global memory: a generic one would make this a flat load, which also counts as
        // an LDS access and would be waited for with the kernel arguments)
        ph[i] = *(const __attribute__((address_space(1))) uint32_t*)pv;
    }
}

template <int NL>
__device__ __forceinline__ void mark_pixel(const MarkSetN<NL>& mk, const uint32_t (&ph)[NL > 0 ? NL : 1], int py, int px)
{
#pragma unroll
    for (int i = 0; i < NL; ++i)
        if (i < mk.n) mark_blocks(mk.m[i], ph[i], py, px);
}

// The fields of one list as scalar-register inputs of an empty statement: the compiler then fetches
// them in one batch at the top of the kernel instead of group by group before each first use.
#define SIGE_PIN_MARK(L_)                                                                                          \
    asm volatile("" ::"s"((L_).flags), "s"((L_).half), "s"((L_).pool_log2), "s"((L_).oy), "s"((L_).ox), "s"((L_).hi), \
                 "s"((L_).sy), "s"((L_).sx), "s"((L_).nby), "s"((L_).nbx), "s"((L_).ly), "s"((L_).lx),                  \
                 "s"((L_).dsy.d), "s"((L_).dsy.m), "s"((L_).dsx.d), "s"((L_).dsx.m))

// V = vectors per pixel = 1 << log2v, V <= 64.  One wave covers 64/V pixels per step.
// NL = lists the launch can mark for (0: mask only; the kernel then carries no marking code and no list
// arguments).  Every wave of this kernel lives for one round trip to memory, so what it does before its
// first load counts: the list arguments are fetched in one batch (left to itself the compiler fetches them
// in five or six dependent groups at the top of EVERY wave: +0.7 us for the kernel), and eight waves per
// SIMD are required of the compiler: the launch is sized so that the whole tensor is in flight in one
// round of workgroups, and at seven waves the last eighth runs as a second round (8.1 instead of 6.3 us
// at 33 MB).
template <typename T, int U, int NL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8)))
void diff_mask_pow2(const uint4* __restrict__ a_o, const uint4* __restrict__ a_e, long n_vec, int log2v, float tau,
                    long n_pix, uint8_t* __restrict__ mask, MarkSetN<NL> mk)
{
    // what every wave needs, fetched in one batch
    asm volatile("" ::"s"(a_o), "s"(a_e), "s"(n_vec), "s"(log2v), "s"(tau), "s"(n_pix), "s"(mask));
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int V = 1 << log2v;
    const int ppw = 64 >> log2v;  // pixels per wave step
    const unsigned long long gmask = V == 64 ? ~0ull : ((1ull << V) - 1ull);
    // (one step per wave and no loop around it: the compiler moves whatever a loop leaves unchanged to
    // the front of it, and here that is the marking path's arithmetic, run by every wave for nothing)
    const long base = wave * (64L * U);
    // The phase words of the lists are asked for FIRST, by every wave: loads return in the order they were
    // issued and these hit the cache (one address per list for the whole launch), so they are there before the
    // streamed data and the few lanes that mark do not wait for a second round trip behind it.
    uint32_t ph[NL > 0 ? NL : 1] = {};
    if constexpr (NL > 0) load_phases(mk, ph);       // (an instance with lists is launched only with mk.n >= 1)
    if (base < n_vec) {
        // Unconditional loads at clamped indices, so that all 2U of them are in flight before the first is
        // looked at (with a bounds test around each pair the compiler finishes one pair before it issues the
        // next: U round trips to memory instead of one).  A clamped vector belongs to a pixel >= n_pix,
        // which is not stored below.
        uint4 o[U], e[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long idx = min(base + u * 64 + lane, n_vec - 1);
            o[u] = load_stream(a_o + idx);
            e[u] = load_stream(a_e + idx);
        }
        // (neither the optimiser nor the instruction scheduler may move a load below this point or a use
        // of a loaded value above it)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            unsigned long long b = __ballot(vec_differs<T>(o[u], e[u], tau));
            long pix = ((base + u * 64) >> log2v) + lane;
            if (lane < ppw && pix < n_pix) {
                const bool marked = ((b >> (lane << log2v)) & gmask) != 0ull;
                mask[pix] = marked ? 1 : 0;
                if constexpr (NL > 0) {
                    if (marked && mk.n) {
                        int py, px;                               // the host checked that pixels fit 31 bits
                        pixel_rc(mk, (int)pix, py, px);
                        mark_pixel(mk, ph, py, px);
                    }
                }
            }
        }
    }
    // (last, so that nothing of it sits in front of the first wave's loads)
    if constexpr (NL > 0)
        if (blockIdx.x == 0 && threadIdx.x == 0) publish_phase(mk);
}

// Any number of vectors per pixel: one wave per pixel.
template <typename T>
__global__ __launch_bounds__(256) void diff_mask_wave(const uint4* __restrict__ a_o,
                                                      const uint4* __restrict__ a_e, int V, float tau,
                                                      long n_pix, uint8_t* __restrict__ mask)
{
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long n_waves = (long)gridDim.x * (blockDim.x >> 6);
    for (long pix = wave; pix < n_pix; pix += n_waves) {
        bool any = false;
        for (int j = lane; j < V; j += 64)
            any |= vec_differs<T>(a_o[pix * V + j], a_e[pix * V + j], tau);
        unsigned long long b = __ballot(any);
        if (lane == 0) mask[pix] = b ? 1 : 0;
    }
}

// Channel counts whose pixel is not a whole number of 16-byte vectors: one thread per pixel.
template <typename T>
__global__ __launch_bounds__(256) void diff_mask_scalar(const T* __restrict__ a_o,
                                                        const T* __restrict__ a_e, int C, float tau,
                                                        long n_pix, uint8_t* __restrict__ mask)
{
    long pix = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= n_pix) return;
    bool any = false;
    for (int c = 0; c < C; ++c)
        any |= !(fabsf(to_f32(a_e[pix * C + c]) - to_f32(a_o[pix * C + c])) <= tau);
    mask[pix] = any ? 1 : 0;
}

struct ListArgs {
    const uint8_t* mask;
    int Hm, Wm, pool_log2, dilate;
    int Hin, Win, bh, bw, stride, pad, th, tw;
    int nby, nbx;
    int32_t* indices;
    int max_blocks;
    int32_t* count;
    int words;  // 1: pooled windows may be read as aligned 32-bit words
};

// True iff the input tile of block blk (clipped to the image, grown by the dilation radius)
// holds a marked pixel of the pooled mask.  Evaluated by one whole wave.
__device__ __forceinline__ bool block_is_active(const ListArgs& a, int blk, int lane)
{
    const int p = a.pool_log2;
    const int by = blk / a.nbx, bx = blk - by * a.nbx;
    int fy0 = by * a.bh * a.stride - a.pad, fx0 = bx * a.bw * a.stride - a.pad;
    int fy1 = min(fy0 + a.th, a.Hin), fx1 = min(fx0 + a.tw, a.Win);
    fy0 = max(fy0, 0);
    fx0 = max(fx0, 0);
    const int ry0 = max(fy0 - a.dilate, 0), ry1 = min(fy1 + a.dilate, a.Hin);
    const int rx0 = max(fx0 - a.dilate, 0), rx1 = min(fx1 + a.dilate, a.Win);
    const int ncols = rx1 - rx0, n = (ry1 - ry0) * ncols;
    bool any = false;
    for (int e = lane; e < n; e += 64) {
        const int y = ry0 + e / ncols, x = rx0 + e % ncols;
        if (p == 0) {
            any |= a.mask[(long)y * a.Wm + x] != 0;
        } else {
            const int sy1 = min((y + 1) << p, a.Hm), sx0 = x << p, sx1 = min((x + 1) << p, a.Wm);
            for (int sy = y << p; sy < sy1; ++sy) {
                if (a.words) {
                    const uint32_t* row = reinterpret_cast<const uint32_t*>(a.mask + (long)sy * a.Wm);
                    for (int sx = sx0 >> 2; sx < (sx1 >> 2); ++sx) any |= row[sx] != 0;
                } else {
                    for (int sx = sx0; sx < sx1; ++sx) any |= a.mask[(long)sy * a.Wm + sx] != 0;
                }
            }
        }
    }
    return __ballot(any) != 0ull;
}

// Ordered compaction of nb flags by one workgroup of NT threads: blocks are visited in
// row-major order, NT at a time; ballot + popcount give the position inside a wave, the wave
// totals are scanned through LDS.
template <int NT>
__device__ __forceinline__ void compact_flags(const ListArgs& a, const uint8_t* flags, int nb, int* wave_tot)
{
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int base = 0;
    for (int c0 = 0; c0 < nb; c0 += NT) {
        const int blk = c0 + tid;
        const int f = blk < nb ? flags[blk] : 0;
        const unsigned long long b = __ballot(f);
        const int pre = __popcll(b & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[w] = __popcll(b);
        __syncthreads();
        int off = base, total = 0;
        for (int i = 0; i < NW; ++i) {
            const int t = wave_tot[i];
            if (i < w) off += t;
            total += t;
        }
        if (f) {
            const int slot = off + pre;
            if (slot < a.max_blocks) {
                const int by = blk / a.nbx;
                a.indices[2 * slot] = by * a.bh;
                a.indices[2 * slot + 1] = (blk - by * a.nbx) * a.bw;
            }
        }
        base += total;
        __syncthreads();
    }
    if (tid == 0) *a.count = base;
}

// Ready mask -> block flags: every lane reads 4 mask bytes of one row and marks for the non-zero
// ones (32-bit index arithmetic only; the few marked pixels are spread over many lanes).
__global__ __launch_bounds__(256) void mark_from_mask_kernel(const uint8_t* __restrict__ mask, int Hm,
                                                             int words_per_row, int aligned, MarkSet mk)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) publish_phase(mk);
    if (t >= Hm * words_per_row) return;
    uint32_t ph[MAX_LISTS];
    load_phases(mk, ph);
    const int Wm = mk.Wm;
    const int y = t / words_per_row, x0 = (t - y * words_per_row) * 4;
    const uint8_t* row = mask + (long)y * Wm;
    if (aligned && x0 + 4 <= Wm) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(row + x0);
        if (w == 0u) return;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if ((w >> (8 * j)) & 0xffu)
                mark_pixel(mk, ph, y, x0 + j);
    } else {
        for (int x = x0; x < min(x0 + 4, Wm); ++x)
            if (row[x])
                mark_pixel(mk, ph, y, x);
    }
}

struct ListSet {
    ListArgs a[MAX_LISTS];
    uint8_t* flags[MAX_LISTS];   // the flag workspaces (two halves, phase words)
    int half[MAX_LISTS];
};

// Flags (global) -> ordered list, one workgroup per list; the flags are cleared again for the
// next call.
__global__ __launch_bounds__(1024) void compact_ws_kernel(ListSet s)
{
    __shared__ int wave_tot[16];
    const ListArgs& a = s.a[blockIdx.x];
    const int half = s.half[blockIdx.x];
    uint8_t* flags = s.flags[blockIdx.x] + (phase_of(s.flags[blockIdx.x], half) & 1u) * half;
    const int nb = a.nby * a.nbx;
    compact_flags<1024>(a, flags, nb, wave_tot);
    for (int i = threadIdx.x; i < nb; i += 1024) flags[i] = 0;
}

// Without a workspace: one workgroup tests every block (flags in LDS) and compacts.
__global__ __launch_bounds__(1024) void block_list_kernel(ListArgs a)
{
    extern __shared__ uint8_t flags[];
    __shared__ int wave_tot[16];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int nb = a.nby * a.nbx;
    for (int blk = w; blk < nb; blk += 16) {
        const bool f = block_is_active(a, blk, lane);
        if (lane == 0) flags[blk] = f ? 1 : 0;
    }
    __syncthreads();
    compact_flags<1024>(a, flags, nb, wave_tot);
}

template <typename T>
static int launch_diff(const void* a_orig, const void* a_edit, int Hm, int Wm, int C, float tau,
                       uint8_t* mask, const MarkSet& mk, bool* marked, hipStream_t st)
{
    *marked = false;
    const long n_pix = (long)Hm * Wm;
    const size_t bytes = (size_t)C * sizeof(T);
    if (bytes % 16 == 0 && aligned16(a_orig) && aligned16(a_edit)) {
        const int V = (int)(bytes / 16);
        const long n_vec = n_pix * V;
        if (V <= 64 && (V & (V - 1)) == 0) {
            int log2v = 0;
            while ((1 << log2v) < V) ++log2v;
            // two 16-byte loads per tensor and lane in flight, one step per workgroup up to 32768 workgroups
            // (measured: 7.3 - 7.5 us at 32 MB whatever the grain between 1024 and 8192 workgroups and 1 - 2
            // loads, 8.3 us with 4 loads, 11.7 us with 8; at 512 MB 77 us with 32768 workgroups, 81 us with 8192)
            const int U = knob(SIGE_KNOB_DIFF_LOADS) > 0 ? knob(SIGE_KNOB_DIFF_LOADS) : 2;
            const long steps = (n_vec + 256L * U - 1) / (256L * U);     // one step per wave
            SIGE_REQUIRE(steps < (1L << 24), SIGE_ERR_UNSUPPORTED, "sige_reduce_mask: more than 2^32 threads");
            const int grid = (int)steps;
            // the kernel instance that carries just as many lists as the call has (0, 1, 2 or up to MAX_LISTS)
            auto launch_n = [&](auto nl_c) {
                constexpr int NL = decltype(nl_c)::value;
                MarkSetN<NL> mn;
                mn.n = mk.n; mn.Wm = mk.Wm; mn.lW = mk.lW; mn.dWm = mk.dWm;
                for (int i = 0; i < NL && i < mk.n; ++i) mn.m[i] = mk.m[i];
                auto launch = [&](auto kern) {
                    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, st, (const uint4*)a_orig, (const uint4*)a_edit,
                                       n_vec, log2v, tau, n_pix, mask, mn);
                };
                if (U == 1) launch(diff_mask_pow2<T, 1, NL>);
                else if (U == 4) launch(diff_mask_pow2<T, 4, NL>);
                else launch(diff_mask_pow2<T, 2, NL>);
            };
            if (mk.n == 0) launch_n(std::integral_constant<int, 0>{});
            else if (mk.n == 1) launch_n(std::integral_constant<int, 1>{});
            else if (mk.n == 2) launch_n(std::integral_constant<int, 2>{});
            else launch_n(std::integral_constant<int, MAX_LISTS>{});
            *marked = mk.n != 0;
        } else {
            long blocks = (n_pix + 3) / 4;
            int grid = (int)(blocks < 8192 ? blocks : 8192);
            hipLaunchKernelGGL((diff_mask_wave<T>), dim3(grid), dim3(256), 0, st, (const uint4*)a_orig,
                               (const uint4*)a_edit, V, tau, n_pix, mask);
        }
    } else {
        long blocks = (n_pix + 255) / 256;
        SIGE_REQUIRE(blocks < (1L << 31), SIGE_ERR_UNSUPPORTED, "sige_reduce_mask: mask too large");
        hipLaunchKernelGGL((diff_mask_scalar<T>), dim3((int)blocks), dim3(256), 0, st, (const T*)a_orig,
                           (const T*)a_edit, C, tau, n_pix, mask);
    }
    SIGE_LAUNCH_CHECK("sige_reduce_mask(diff)");
    return SIGE_OK;
}

// The second half of a reduction whose first half was sige_mark_blocks: flags -> ordered lists, flags cleared.
int compact_marked_lists(const char* who, const sige_block_list* lists, int n, hipStream_t st)
{
    SIGE_REQUIRE(n >= 1 && n <= MAX_LISTS, SIGE_ERR_INVALID_ARG, "%s: between 1 and %d lists", who, MAX_LISTS);
    ListSet ls;
    for (int i = 0; i < n; ++i) {
        const sige_geom* g = &lists[i].g;
        ListArgs& a = ls.a[i];
        a = ListArgs{};
        a.bh = g->block_h; a.bw = g->block_w;
        a.nby = (g->H_out + g->block_h - 1) / g->block_h;
        a.nbx = (g->W_out + g->block_w - 1) / g->block_w;
        a.indices = lists[i].indices; a.max_blocks = lists[i].max_blocks; a.count = lists[i].count;
        ls.flags[i] = (uint8_t*)lists[i].workspace;
        ls.half[i] = (a.nby * a.nbx + 15) & ~15;
    }
    hipLaunchKernelGGL(compact_ws_kernel, dim3(n), dim3(1024), 0, st, ls);
    SIGE_LAUNCH_CHECK(who);
    return SIGE_OK;
}

}  // namespace sige

using namespace sige;

extern "C" size_t sige_reduce_mask_workspace_bytes(const sige_geom* g)
{
    if (g == nullptr || g->block_h <= 0 || g->block_w <= 0 || g->H_out <= 0 || g->W_out <= 0) return 0;
    const size_t nb = (size_t)((g->H_out + g->block_h - 1) / g->block_h) * ((g->W_out + g->block_w - 1) / g->block_w);
    // two halves of one flag per block, then the phase words
    return 2 * ((nb + 15) & ~(size_t)15) + 16;
}

// Shared by both entry points: n lists (n >= 1; n == 0 only for the mask-only mode) built from one
// mask.  With n == 1 a missing workspace falls back to the single-workgroup block test.
static int reduce_lists(const char* who, const void* a_orig, const void* a_edit, sige_dtype dt, int32_t Hm,
                        int32_t Wm, int32_t C, float tau, const uint8_t* mask_in, int32_t pool_log2,
                        int32_t dilate, const sige_block_list* lists, int n, const sige_geom* g_mask_only,
                        uint8_t* mask_out, void* stream, bool mark_only = false)
{
    const bool diff_mode = a_orig != nullptr || a_edit != nullptr;
    SIGE_REQUIRE(diff_mode != (mask_in != nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: give either (a_orig, a_edit) or mask_in, not both and not neither", who);
    SIGE_REQUIRE(Hm > 0 && Wm > 0, SIGE_ERR_INVALID_ARG, "%s: mask size must be positive", who);
    SIGE_REQUIRE((long)Hm * Wm < (1L << 31), SIGE_ERR_UNSUPPORTED, "%s: mask larger than 2^31 pixels", who);
    SIGE_REQUIRE(pool_log2 >= 0 && pool_log2 <= 12 && dilate >= 0, SIGE_ERR_INVALID_ARG,
                 "%s: pool_log2 must be in [0, 12] and dilate >= 0", who);
    const int ps = 1 << pool_log2;
    const int Hp = (Hm + ps - 1) / ps, Wp = (Wm + ps - 1) / ps;
    hipStream_t st = (hipStream_t)stream;
    auto log2_or = [](int v) { int l = 0; while ((1 << l) < v) ++l; return (1 << l) == v ? l : -1; };
    MarkSet mk;
    mk.n = 0;
    mk.Wm = Wm; mk.lW = log2_or(Wm); mk.dWm = fast_div(Wm);
    ListSet ls;
    bool all_ws = n > 0;
    for (int i = 0; i < n; ++i) {
        const sige_block_list& L = lists[i];
        const sige_geom* g = &L.g;
        int th, tw;
        if (int rc = check_geom(g, who, &th, &tw)) return rc;
        SIGE_REQUIRE(Hp == g->H_in && Wp == g->W_in, SIGE_ERR_INVALID_ARG,
                     "%s: pooled mask %dx%d does not match the conv input %dx%d", who, Hp, Wp, g->H_in, g->W_in);
        SIGE_REQUIRE(L.indices != nullptr && L.count != nullptr, SIGE_ERR_INVALID_ARG,
                     "%s: indices and count are required (both NULL only to get just the difference mask)", who);
        SIGE_REQUIRE(L.max_blocks >= 0, SIGE_ERR_INVALID_ARG, "%s: max_blocks is negative", who);
        const long nby = (g->H_out + g->block_h - 1) / g->block_h, nbx = (g->W_out + g->block_w - 1) / g->block_w;
        SIGE_REQUIRE(nby * nbx <= 131072, SIGE_ERR_CAPACITY, "%s: block grid %ldx%ld exceeds 131072 blocks", who,
                     nby, nbx);
        const bool ws = L.workspace != nullptr && L.workspace_bytes >= sige_reduce_mask_workspace_bytes(g) &&
                        (reinterpret_cast<uintptr_t>(L.workspace) & 15u) == 0;
        all_ws = all_ws && ws;
        for (int j = 0; j < i; ++j)
            SIGE_REQUIRE(!ws || lists[j].workspace != L.workspace, SIGE_ERR_INVALID_ARG,
                         "%s: lists %d and %d share a workspace", who, j, i);
        MarkArgs& m = mk.m[i];
        m.flags = (uint8_t*)L.workspace;
        m.half = (int)((nby * nbx + 15) & ~15L);
        m.pool_log2 = pool_log2;
        m.oy = dilate + th - g->pad; m.ox = dilate + tw - g->pad; m.hi = dilate + g->pad;
        m.sy = g->block_h * g->stride; m.sx = g->block_w * g->stride;
        m.nby = (int)nby; m.nbx = (int)nbx;
        m.dsy = fast_div(m.sy); m.dsx = fast_div(m.sx);
        m.ly = log2_or(m.sy); m.lx = log2_or(m.sx);
        ListArgs& a = ls.a[i];
        a.Hm = Hm; a.Wm = Wm; a.pool_log2 = pool_log2; a.dilate = dilate;
        a.Hin = g->H_in; a.Win = g->W_in; a.bh = g->block_h; a.bw = g->block_w;
        a.stride = g->stride; a.pad = g->pad; a.th = th; a.tw = tw;
        a.nby = (int)nby; a.nbx = (int)nbx;
        a.indices = L.indices; a.max_blocks = L.max_blocks; a.count = L.count;
        ls.flags[i] = (uint8_t*)L.workspace;
        ls.half[i] = m.half;
    }
    SIGE_REQUIRE(n <= 1 || all_ws, SIGE_ERR_INVALID_ARG,
                 "%s: every list needs its own zeroed, 16-byte aligned workspace of "
                 "sige_reduce_mask_workspace_bytes(g) bytes", who);
    if (n == 0) {   // mask only: the geometry only has to match the pooled size
        int th, tw;
        if (int rc = check_geom(g_mask_only, who, &th, &tw)) return rc;
        SIGE_REQUIRE(Hp == g_mask_only->H_in && Wp == g_mask_only->W_in, SIGE_ERR_INVALID_ARG,
                     "%s: pooled mask %dx%d does not match the conv input %dx%d", who, Hp, Wp,
                     g_mask_only->H_in, g_mask_only->W_in);
    }
    if (all_ws) mk.n = n;
    const uint8_t* mask = mask_in;
    bool marked = false;
    if (diff_mode) {
        SIGE_REQUIRE(a_orig && a_edit, SIGE_ERR_INVALID_ARG, "%s: a_orig and a_edit are both required", who);
        SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
        SIGE_REQUIRE(C > 0, SIGE_ERR_INVALID_ARG, "%s: C must be positive", who);
        SIGE_REQUIRE(mask_out != nullptr, SIGE_ERR_INVALID_ARG,
                     "%s: mask_out is required when the mask is computed from activations", who);
        int rc = dt == SIGE_F32   ? launch_diff<float>(a_orig, a_edit, Hm, Wm, C, tau, mask_out, mk, &marked, st)
                 : dt == SIGE_F16 ? launch_diff<f16>(a_orig, a_edit, Hm, Wm, C, tau, mask_out, mk, &marked, st)
                                  : launch_diff<bf16>(a_orig, a_edit, Hm, Wm, C, tau, mask_out, mk, &marked, st);
        if (rc) return rc;
        mask = mask_out;
        if (n == 0) return SIGE_OK;
    }
    const int words = (pool_log2 >= 2 && Wm % 4 == 0 && (reinterpret_cast<uintptr_t>(mask) & 3u) == 0) ? 1 : 0;
    for (int i = 0; i < n; ++i) { ls.a[i].mask = mask; ls.a[i].words = words; }
    if (all_ws) {
        if (!marked) {
            const int wpr = (Wm + 3) / 4;
            const long threads = (long)Hm * wpr;
            const int aligned = (reinterpret_cast<uintptr_t>(mask) & 3u) == 0 && Wm % 4 == 0;
            hipLaunchKernelGGL(mark_from_mask_kernel, dim3((int)((threads + 255) / 256)), dim3(256), 0, st, mask,
                               Hm, wpr, aligned, mk);
            SIGE_LAUNCH_CHECK("sige_reduce_mask(mark)");
        }
        if (mark_only) return SIGE_OK;     // the consumer of the marked lists compacts
        hipLaunchKernelGGL(compact_ws_kernel, dim3(n), dim3(1024), 0, st, ls);
        SIGE_LAUNCH_CHECK("sige_reduce_mask(compact)");
        return SIGE_OK;
    }
    SIGE_REQUIRE(!mark_only, SIGE_ERR_INVALID_ARG, "%s: every list needs its flag workspace", who);
    const ListArgs& a = ls.a[0];
    const size_t lds = ((size_t)(a.nby * a.nbx) + 15) & ~(size_t)15;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)block_list_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "%s: cannot reserve %zu bytes of LDS: %s", who, lds,
                     hipGetErrorString(e));
    }
    hipLaunchKernelGGL(block_list_kernel, dim3(1), dim3(1024), lds, st, a);
    SIGE_LAUNCH_CHECK("sige_reduce_mask(list)");
    return SIGE_OK;
}

extern "C" int sige_reduce_mask(const void* a_orig, const void* a_edit, sige_dtype dt, int32_t Hm,
                                int32_t Wm, int32_t C, float tau, const uint8_t* mask_in,
                                int32_t pool_log2, int32_t dilate, const sige_geom* g,
                                uint8_t* mask_out, int32_t* indices, int32_t max_blocks,
                                int32_t* count, void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    const char* who = "sige_reduce_mask";
    SIGE_REQUIRE(g != nullptr, SIGE_ERR_INVALID_ARG, "%s: geometry is NULL", who);
    const bool diff_mode = a_orig != nullptr || a_edit != nullptr;
    if (diff_mode && indices == nullptr && count == nullptr)
        return reduce_lists(who, a_orig, a_edit, dt, Hm, Wm, C, tau, mask_in, pool_log2, dilate, nullptr, 0, g,
                            mask_out, stream);
    sige_block_list L;
    L.g = *g; L.indices = indices; L.max_blocks = max_blocks; L.count = count;
    L.workspace = workspace; L.workspace_bytes = workspace_bytes;
    return reduce_lists(who, a_orig, a_edit, dt, Hm, Wm, C, tau, mask_in, pool_log2, dilate, &L, 1, nullptr,
                        mask_out, stream);
}

// ---- the same reduction for callers that cannot allocate ------------------------------------------
// The block flags live in a file-scope device array instead of a caller workspace.  In host code the
// array's name is only a stand-in for the symbol: the address the kernels get is resolved once per
// device with hipGetSymbolAddress (each GPU holds its own copy at its own address) and kept.
static __device__ __align__(256) unsigned char scratch[2 * SIGE_NOALLOC_MAX_BLOCKS + 16];

namespace sige {

__global__ __launch_bounds__(256) void clear_scratch_kernel(uint4* p, int n_vec)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n_vec) p[i] = make_uint4(0, 0, 0, 0);
}

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];      // per device, nullptr until resolved
static std::mutex g_scratch_mutex;

// The device address of `scratch` on the current device; the first time on a device the whole
// array is cleared by a small kernel on `st` (the reduction's kernels follow on the same stream).
static int scratch_address(const char* who, hipStream_t st, void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    SIGE_REQUIRE(e == hipSuccess, SIGE_ERR_HIP, "%s: hipGetDevice: %s", who, hipGetErrorString(e));
    SIGE_REQUIRE(dev >= 0 && dev < kMaxDevices, SIGE_ERR_UNSUPPORTED, "%s: device ordinal %d beyond %d", who, dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        SIGE_REQUIRE(e == hipSuccess && ptr != nullptr, SIGE_ERR_HIP, "%s: hipGetSymbolAddress: %s", who,
                     hipGetErrorString(e));
        constexpr int n_vec = (2 * SIGE_NOALLOC_MAX_BLOCKS + 16) / 16;
        hipLaunchKernelGGL(clear_scratch_kernel, dim3((n_vec + 255) / 256), dim3(256), 0, st, (uint4*)ptr, n_vec);
        SIGE_LAUNCH_CHECK(who);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SIGE_OK;
}

}  // namespace sige

extern "C" int sige_reduce_mask_noalloc(const void* a_orig, const void* a_edit, sige_dtype dt, int32_t Hm,
                                        int32_t Wm, int32_t C, float tau, const uint8_t* mask_in,
                                        int32_t pool_log2, int32_t dilate, const sige_geom* g,
                                        uint8_t* mask_out, int32_t* indices, int32_t max_blocks,
                                        int32_t* count, void* stream)
{
    clear_error();
    const char* who = "sige_reduce_mask_noalloc";
    SIGE_REQUIRE(g != nullptr, SIGE_ERR_INVALID_ARG, "%s: geometry is NULL", who);
    int th, tw;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    SIGE_REQUIRE(indices != nullptr && count != nullptr, SIGE_ERR_INVALID_ARG, "%s: indices and count are required", who);
    const size_t need = sige_reduce_mask_workspace_bytes(g);
    SIGE_REQUIRE(need <= 2 * (size_t)SIGE_NOALLOC_MAX_BLOCKS + 16, SIGE_ERR_CAPACITY,
                 "%s: the block grid has %zu blocks, the built-in scratch holds %d", who,
                 (size_t)((g->H_out + g->block_h - 1) / g->block_h) * ((g->W_out + g->block_w - 1) / g->block_w),
                 SIGE_NOALLOC_MAX_BLOCKS);
    // every other argument error is found before the device is touched
    const bool diff_mode = a_orig != nullptr || a_edit != nullptr;
    SIGE_REQUIRE(diff_mode != (mask_in != nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: give either (a_orig, a_edit) or mask_in, not both and not neither", who);
    SIGE_REQUIRE(!diff_mode || (a_orig && a_edit && mask_out), SIGE_ERR_INVALID_ARG,
                 "%s: a_orig, a_edit and mask_out are required when the mask is computed from activations", who);
    SIGE_REQUIRE(max_blocks >= 0, SIGE_ERR_INVALID_ARG, "%s: max_blocks is negative", who);
    void* ptr = nullptr;
    if (int rc = scratch_address(who, (hipStream_t)stream, &ptr)) return rc;
    sige_block_list L;
    L.g = *g; L.indices = indices; L.max_blocks = max_blocks; L.count = count;
    L.workspace = ptr; L.workspace_bytes = need;
    return reduce_lists(who, a_orig, a_edit, dt, Hm, Wm, C, tau, mask_in, pool_log2, dilate, &L, 1, nullptr,
                        mask_out, stream);
}

extern "C" int sige_reduce_mask_lists(const void* a_orig, const void* a_edit, sige_dtype dt, int32_t Hm,
                                      int32_t Wm, int32_t C, float tau, const uint8_t* mask_in,
                                      int32_t pool_log2, int32_t dilate, const sige_block_list* lists,
                                      int32_t n_lists, uint8_t* mask_out, void* stream)
{
    clear_error();
    const char* who = "sige_reduce_mask_lists";
    SIGE_REQUIRE(lists != nullptr && n_lists >= 1 && n_lists <= MAX_LISTS, SIGE_ERR_INVALID_ARG,
                 "%s: between 1 and %d lists per call", who, MAX_LISTS);
    for (int i = 0; i < n_lists; ++i)
        SIGE_REQUIRE(lists[i].workspace != nullptr, SIGE_ERR_INVALID_ARG, "%s: list %d has no workspace", who, i);
    return reduce_lists(who, a_orig, a_edit, dt, Hm, Wm, C, tau, mask_in, pool_log2, dilate, lists, n_lists,
                        nullptr, mask_out, stream);
}

extern "C" int sige_mark_blocks(const void* a_orig, const void* a_edit, sige_dtype dt, int32_t Hm, int32_t Wm,
                                int32_t C, float tau, const uint8_t* mask_in, int32_t pool_log2, int32_t dilate,
                                const sige_block_list* lists, int32_t n_lists, uint8_t* mask_out, void* stream)
{
    clear_error();
    const char* who = "sige_mark_blocks";
    SIGE_REQUIRE(lists != nullptr && n_lists >= 1 && n_lists <= MAX_LISTS, SIGE_ERR_INVALID_ARG,
                 "%s: between 1 and %d lists per call", who, MAX_LISTS);
    for (int i = 0; i < n_lists; ++i)
        SIGE_REQUIRE(lists[i].workspace != nullptr, SIGE_ERR_INVALID_ARG, "%s: list %d has no workspace", who, i);
    return reduce_lists(who, a_orig, a_edit, dt, Hm, Wm, C, tau, mask_in, pool_log2, dilate, lists, n_lists,
                        nullptr, mask_out, stream, true);
}
