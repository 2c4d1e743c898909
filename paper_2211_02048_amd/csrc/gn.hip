// sige_gn_stats: group statistics of a full tensor, folded into the per-channel
// Scale+Shift that replaces the normalisation layer once the statistics of the
// original activation are cached (Sec. 3.2 "Pre-computing normalization parameters").
// Used by the pre-computation pass, and by the sparse pass of a generator at the low resolutions
// whose statistics are recomputed instead of cached (Sec. 4.1).
//
// Small tensors (the low resolutions): ONE kernel, each workgroup owns the channels of a few whole
// groups, sums them over all pixels in a fixed order (no atomics: the result is reproducible bit for
// bit) and writes mean, variance, scale and shift itself.
// Large tensors: pass 1 streams the tensor once, fully coalesced (every lane keeps one 16-byte
// channel group and walks down the pixels), reduces per-group sums of x and x^2 in
// LDS and adds them to the fp32 accumulators; pass 2 (one workgroup) turns the sums
// into mean / biased variance and the folded scale and shift.
#include "common.h"

namespace sige {

__global__ void gn_zero_kernel(float* mean, float* var, int groups)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < groups) { mean[i] = 0.0f; var[i] = 0.0f; }
}

// Adds one lane's per-channel sums (channels cgv*N .. cgv*N+N-1) to the per-group sums in LDS,
// combining the channels of one group in registers first where the group size allows.
template <int N>
__device__ __forceinline__ void add_to_groups(float* red, int groups, int cgv, int cg, const float (&s)[N],
                                              const float (&q)[N])
{
    if (cg % N == 0) {                       // the vector lies inside one group
        float st = 0.0f, qt = 0.0f;
#pragma unroll
        for (int i = 0; i < N; ++i) { st += s[i]; qt += q[i]; }
        const int g = cgv * N / cg;
        atomicAdd(&red[g], st);
        atomicAdd(&red[groups + g], qt);
    } else if (N % cg == 0) {                // the vector holds N / cg whole groups
        float st = 0.0f, qt = 0.0f;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            st += s[i];
            qt += q[i];
            if ((i + 1) % cg == 0) {
                const int g = (cgv * N + i) / cg;
                atomicAdd(&red[g], st);
                atomicAdd(&red[groups + g], qt);
                st = 0.0f;
                qt = 0.0f;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int g = (cgv * N + i) / cg;
            atomicAdd(&red[g], s[i]);
            atomicAdd(&red[groups + g], q[i]);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gn_sum_kernel(const uint4* __restrict__ x, long n_pix, int V,
                                                     int ld_vec, int cg, int groups,
                                                     float* __restrict__ sum, float* __restrict__ sumsq)
{
    constexpr int N = Vec16<T>::N;
    constexpr int U = 4;            // loads in flight per lane
    extern __shared__ float red[];  // [2][groups]
    for (int i = threadIdx.x; i < 2 * groups; i += 256) red[i] = 0.0f;
    __syncthreads();
    // Up to 256 vectors per pixel: the first (256 / V) * V threads each keep one channel group and
    // walk down the pixels (the rest idle, none when V divides 256).
    if (V <= 256) {
        const int cgv = threadIdx.x % V, ppi = 256 / V;  // pixels per workgroup step
        const bool active = threadIdx.x < ppi * V;
        float s[N], q[N];
#pragma unroll
        for (int i = 0; i < N; ++i) { s[i] = 0.0f; q[i] = 0.0f; }
        const long stride = (long)gridDim.x * ppi;
        for (long p = (long)blockIdx.x * ppi + threadIdx.x / V; active && p < n_pix; p += U * stride) {
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long pp = p + u * stride;
                v[u] = pp < n_pix ? x[pp * ld_vec + cgv] : make_uint4(0, 0, 0, 0);   // zeros add nothing
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float f[N];
                unpack<T>(v[u], f);
#pragma unroll
                for (int i = 0; i < N; ++i) { s[i] += f[i]; q[i] = fmaf(f[i], f[i], q[i]); }
            }
        }
        // lanes of a wave that hold the same channel group are V apart: when V is a power of two below
        // 64, fold them onto the first V lanes, which then add to LDS
        if (V < 64 && (V & (V - 1)) == 0) {
            for (int off = V; off < 64; off <<= 1)
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    s[i] += __shfl_xor(s[i], off);
                    q[i] += __shfl_xor(q[i], off);
                }
            if ((threadIdx.x & 63) < V) add_to_groups<N>(red, groups, cgv, cg, s, q);
        } else if (active) {
            add_to_groups<N>(red, groups, cgv, cg, s, q);
        }
    } else {
        const long n_vec = n_pix * V;
        for (long j = (long)blockIdx.x * 256 + threadIdx.x; j < n_vec; j += (long)gridDim.x * 256) {
            const long p = j / V;
            const int cgv = (int)(j - p * V);
            float f[N], q[N];
            unpack<T>(x[p * ld_vec + cgv], f);
#pragma unroll
            for (int i = 0; i < N; ++i) q[i] = f[i] * f[i];
            add_to_groups<N>(red, groups, cgv, cg, f, q);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < groups; i += 256) {
        atomicAdd(&sum[i], red[i]);
        atomicAdd(&sumsq[i], red[groups + i]);
    }
}

__global__ __launch_bounds__(256) void gn_fold_kernel(float* mean, float* var, float n, int C, int cg,
                                                      int groups, const float* gamma, const float* beta,
                                                      float eps, float* scale, float* shift)
{
    extern __shared__ float st[];  // [2][groups]: mean, var
    for (int g = threadIdx.x; g < groups; g += 256) {
        const float mu = mean[g] / n;
        const float v = fmaxf(var[g] / n - mu * mu, 0.0f);
        st[g] = mu;
        st[groups + g] = v;
    }
    __syncthreads();
    for (int g = threadIdx.x; g < groups; g += 256) { mean[g] = st[g]; var[g] = st[groups + g]; }
    if (scale) {
        for (int c = threadIdx.x; c < C; c += 256) {
            const int g = c / cg;
            const float sc = (gamma ? gamma[c] : 1.0f) * rsqrtf(st[groups + g] + eps);
            scale[c] = sc;
            shift[c] = (beta ? beta[c] : 0.0f) - st[g] * sc;
        }
    }
}

// One workgroup = VW channel vectors (VW * N channels, a whole number of groups) x 256 / VW pixel
// lanes.  Every lane sums its pixels, the lanes' sums meet in LDS and are added in lane order, the
// channels of a group likewise.
template <typename T>
// ppl = 256 / VW pixel lanes, strips = 256 / CW, per = ceil(ppl / strips), gpw = CW / cg groups per
// workgroup and the reciprocals of VW, CW and cg come from the host.
__global__ __launch_bounds__(256) void gn_small_kernel(const uint4* __restrict__ x, int n_pix, int ld_vec, int VW,
                                                       int cg, int ppl, int strips, int per, int gpw,
                                                       FastDiv d_vw, FastDiv d_cw, FastDiv d_cg,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta, float eps,
                                                       float* __restrict__ mean, float* __restrict__ var,
                                                       float* __restrict__ scale, float* __restrict__ shift)
{
    constexpr int N = Vec16<T>::N;
    constexpr int U = 4;               // loads in flight per lane
    extern __shared__ float red[];     // [2][ppl][CW] sums and sums of squares, then [2][CW] mean and variance
    const int CW = VW * N;
    int cv, pl;
    divmod(threadIdx.x, d_vw, pl, cv);
    const int v0 = blockIdx.x * VW;    // first channel vector of this workgroup
    float* sq = red + ppl * CW;
    float* stat = red + 2 * ppl * CW;
    if (pl < ppl) {
        float s[N], q[N];
#pragma unroll
        for (int i = 0; i < N; ++i) { s[i] = 0.0f; q[i] = 0.0f; }
        for (int p = pl; p < n_pix; p += U * ppl) {
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int pp = p + u * ppl;
                v[u] = pp < n_pix ? x[(long)pp * ld_vec + v0 + cv] : make_uint4(0, 0, 0, 0);   // zeros add nothing
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float f[N];
                unpack<T>(v[u], f);
#pragma unroll
                for (int i = 0; i < N; ++i) { s[i] += f[i]; q[i] = fmaf(f[i], f[i], q[i]); }
            }
        }
#pragma unroll
        for (int i = 0; i < N; ++i) {
            red[pl * CW + cv * N + i] = s[i];
            sq[pl * CW + cv * N + i] = q[i];
        }
    }
    __syncthreads();
    // Column sums in two steps, both in a fixed order: 256 / CW threads per channel each add a strip of
    // the pixel lanes, then one thread per channel adds the strips.  (A thread writes only into its
    // own strip's first row, which nobody else reads in that step.)
    {
        int cc, sidx;
        divmod(threadIdx.x, d_cw, sidx, cc);
        if (sidx < strips) {
            const int l0 = sidx * per, l1 = min(l0 + per, ppl);
            float st = 0.0f, qt = 0.0f;
            for (int l = l0; l < l1; ++l) { st += red[l * CW + cc]; qt += sq[l * CW + cc]; }
            if (l0 < ppl) { red[l0 * CW + cc] = st; sq[l0 * CW + cc] = qt; }
        }
    }
    __syncthreads();
    const int c = threadIdx.x;         // channel of the workgroup (c < CW <= 256)
    if (c < CW) {
        float st = 0.0f, qt = 0.0f;
        for (int l0 = 0; l0 < ppl; l0 += per) { st += red[l0 * CW + c]; qt += sq[l0 * CW + c]; }
        red[c] = st;
        sq[c] = qt;
    }
    __syncthreads();
    if (c < gpw) {                     // group c of the workgroup (gpw = CW / cg of them)
        float st = 0.0f, qt = 0.0f;
        for (int j = 0; j < cg; ++j) { st += red[c * cg + j]; qt += sq[c * cg + j]; }
        const float n = (float)n_pix * (float)cg;
        const float mu = st / n;
        const float v = fmaxf(qt / n - mu * mu, 0.0f);
        const int g = blockIdx.x * gpw + c;
        mean[g] = mu;
        var[g] = v;
        stat[c] = mu;
        stat[CW + c] = v;
    }
    __syncthreads();
    if (scale != nullptr && c < CW) {
        int g, rem_;
        divmod(c, d_cg, g, rem_);
        const int ch = v0 * N + c;
        const float sc = (gamma ? gamma[ch] : 1.0f) * rsqrtf(stat[CW + g] + eps);
        scale[ch] = sc;
        shift[ch] = (beta ? beta[ch] : 0.0f) - stat[g] * sc;
    }
}

static int gcd_int(int a, int b) { return b == 0 ? a : gcd_int(b, a % b); }

// Channel vectors per workgroup for the one-kernel path (a whole number of groups), or 0 when the
// tensor is too large for it: at most 32 pixel iterations per lane.
static int small_path_vectors(long n_pix, int cg, int N)
{
    const int VW = cg / gcd_int(cg, N);      // lcm(cg, N) / N
    if (VW > 32) return 0;
    return n_pix <= 32L * (256 / VW) ? VW : 0;
}

template <typename T>
static void launch_small(const void* x, int n_pix, int V, int ld_vec, int VW, int cg, const float* gamma,
                         const float* beta, float eps, float* mean, float* var, float* scale, float* shift,
                         hipStream_t st)
{
    const int ppl = 256 / VW, CW = VW * Vec16<T>::N, strips = 256 / CW;
    const size_t lds = (size_t)(2 * ppl * CW + 2 * CW) * sizeof(float);
    hipLaunchKernelGGL((gn_small_kernel<T>), dim3(V / VW), dim3(256), lds, st, (const uint4*)x, n_pix, ld_vec, VW,
                       cg, ppl, strips, (ppl + strips - 1) / strips, CW / cg, fast_div(VW), fast_div(CW), fast_div(cg), gamma,
                       beta, eps, mean, var, scale, shift);
}

template <typename T>
static void launch_sum(const void* x, long n_pix, int V, int ld_vec, int cg, int groups, float* mean,
                       float* var, hipStream_t st)
{
    // at most two workgroups per compute unit: every workgroup ends with one atomic per group and
    // statistic on the same few addresses, and each lane keeps four loads in flight
    long want = (n_pix * V + 256L * 8 - 1) / (256L * 8);
    int grid = (int)(want < 1 ? 1 : want > 512 ? 512 : want);
    hipLaunchKernelGGL((gn_sum_kernel<T>), dim3(grid), dim3(256), 2 * groups * sizeof(float), st,
                       (const uint4*)x, n_pix, V, ld_vec, cg, groups, mean, var);
}

}  // namespace sige

using namespace sige;

extern "C" int sige_gn_stats(const void* x, sige_dtype dt, int32_t H, int32_t W, int32_t C, int32_t x_ld,
                             int32_t groups, const float* gamma, const float* beta, float eps,
                             float* mean, float* var, float* scale, float* shift, void* stream)
{
    clear_error();
    const char* who = "sige_gn_stats";
    SIGE_REQUIRE(x && mean && var, SIGE_ERR_INVALID_ARG, "%s: x, mean and var are required", who);
    SIGE_REQUIRE((scale == nullptr) == (shift == nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: scale and shift must be given together", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(H > 0 && W > 0 && C > 0 && groups > 0 && x_ld >= C, SIGE_ERR_INVALID_ARG, "%s: bad shape", who);
    SIGE_REQUIRE(C % groups == 0, SIGE_ERR_INVALID_ARG, "%s: C must be divisible by groups", who);
    SIGE_REQUIRE(groups <= 4096, SIGE_ERR_UNSUPPORTED, "%s: at most 4096 groups", who);
    const size_t s = dtype_size(dt);
    SIGE_REQUIRE((C * s) % 16 == 0 && (x_ld * s) % 16 == 0 && aligned16(x), SIGE_ERR_UNSUPPORTED,
                 "%s: C and x_ld must be multiples of %zu elements and x 16-byte aligned", who, 16 / s);
    hipStream_t st = (hipStream_t)stream;
    const long n_pix = (long)H * W;
    const int V = (int)(C * s / 16), ld_vec = (int)(x_ld * s / 16), cg = C / groups;
    if (const int VW = small_path_vectors(n_pix, cg, (int)(16 / s))) {
        if (dt == SIGE_F32) launch_small<float>(x, (int)n_pix, V, ld_vec, VW, cg, gamma, beta, eps, mean, var, scale, shift, st);
        else if (dt == SIGE_F16) launch_small<f16>(x, (int)n_pix, V, ld_vec, VW, cg, gamma, beta, eps, mean, var, scale, shift, st);
        else launch_small<bf16>(x, (int)n_pix, V, ld_vec, VW, cg, gamma, beta, eps, mean, var, scale, shift, st);
        SIGE_LAUNCH_CHECK("sige_gn_stats(small)");
        return SIGE_OK;
    }
    hipLaunchKernelGGL(gn_zero_kernel, dim3((groups + 255) / 256), dim3(256), 0, st, mean, var, groups);
    SIGE_LAUNCH_CHECK("sige_gn_stats(zero)");
    if (dt == SIGE_F32) launch_sum<float>(x, n_pix, V, ld_vec, cg, groups, mean, var, st);
    else if (dt == SIGE_F16) launch_sum<f16>(x, n_pix, V, ld_vec, cg, groups, mean, var, st);
    else launch_sum<bf16>(x, n_pix, V, ld_vec, cg, groups, mean, var, st);
    SIGE_LAUNCH_CHECK("sige_gn_stats(sum)");
    hipLaunchKernelGGL(gn_fold_kernel, dim3(1), dim3(256), 2 * groups * sizeof(float), st, mean, var,
                       (float)n_pix * (float)cg, C, cg, groups, gamma, beta, eps, scale, shift);
    SIGE_LAUNCH_CHECK("sige_gn_stats(fold)");
    return SIGE_OK;
}
