// Token-wise layers of an attention block on the gathered tokens of the active blocks
// (Sec. 3.2 "Extension to attention layers", Fig. "sige-attention": everything between Gather
// and Scatter sees only the edited tokens): per-token layer normalisation and the gated GELU of
// the feed-forward part of a latent-diffusion transformer block (the paper applies the engine to
// that model, Sec. 4.1 "Models", without describing the block; both are the textbook operators).
//
// A "row" is one token: rows are the pixels of the stacked tiles, [n_rows][C] with a row stride.
// The number of rows is a host value or count * rows_per_count read on the device, as everywhere.
#include "common.h"

namespace sige {

struct RowArgs {
    const void* x;
    void* y;
    const float* gamma;
    const float* beta;
    const int32_t* count;
    int C, x_ld, y_ld;
    int rows_per_count, max_rows, n_host;
    float eps;
    // gather mode (indices != NULL): row r is pixel r % (bh * bw) of block r / (bh * bw) of the
    // [H][W][x_ld] tensor x; a pixel outside the tensor is a row of zeros, as in a gathered tile
    const int32_t* indices;
    int bh, bw, H, W;
    FastDiv d_pb, d_bw;     // bh * bw and bw, prepared on the host
};

__device__ __forceinline__ int effective_rows(const RowArgs& a)
{
    if (a.n_host >= 0) return a.n_host;
    const long r = (long)(*a.count) * a.rows_per_count;
    return (int)(r < a.max_rows ? r : a.max_rows);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// One wave per token; the token's channels stay in registers between the two passes (mean, then
// the centred sum of squares), NV 16-byte vectors per lane at most.
template <typename T, int NV>
__global__ __launch_bounds__(256) void token_norm_kernel(RowArgs a)
{
    constexpr int N = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= effective_rows(a)) return;
    const int V = a.C / N;                                  // vectors per token
    long pixel = row;
    bool inside = true;
    if (a.indices != nullptr) {
        int n, p, py, px;
        divmod(row, a.d_pb, n, p);
        divmod(p, a.d_bw, py, px);
        const int iy = a.indices[2 * n] + py, ix = a.indices[2 * n + 1] + px;
        inside = iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
        pixel = inside ? (long)iy * a.W + ix : 0;
    }
    const uint4* __restrict__ src = (const uint4*)((const T*)a.x + pixel * a.x_ld);
    float f[NV][N], gm[NV][N], bt[NV][N];
    uint4 raw[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int j = lane + 64 * u;
        raw[u] = (inside && j < V) ? src[j] : make_uint4(0, 0, 0, 0);
    }
    // gamma and beta do not depend on the statistics: they are fetched right behind the row, as
    // 16-byte vectors (C is a multiple of N, the arrays come from an allocator: 16-byte aligned or
    // the scalar path)
    const bool gvec = aligned16_dev(a.gamma) && aligned16_dev(a.beta);
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int j = lane + 64 * u;
#pragma unroll
        for (int i = 0; i < N; ++i) { gm[u][i] = 1.0f; bt[u][i] = 0.0f; }
        if (j < V) {
            if (gvec) {
#pragma unroll
                for (int i = 0; i < N; i += 4) {
                    if (a.gamma) {
                        const float4 g4 = *(const float4*)(a.gamma + j * N + i);
                        gm[u][i] = g4.x; gm[u][i + 1] = g4.y; gm[u][i + 2] = g4.z; gm[u][i + 3] = g4.w;
                    }
                    if (a.beta) {
                        const float4 b4 = *(const float4*)(a.beta + j * N + i);
                        bt[u][i] = b4.x; bt[u][i + 1] = b4.y; bt[u][i + 2] = b4.z; bt[u][i + 3] = b4.w;
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    if (a.gamma) gm[u][i] = a.gamma[j * N + i];
                    if (a.beta) bt[u][i] = a.beta[j * N + i];
                }
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int j = lane + 64 * u;
        if (j < V) {
            unpack<T>(raw[u], f[u]);
#pragma unroll
            for (int i = 0; i < N; ++i) s += f[u][i];
        }
    }
    const float mean = wave_sum(s) / (float)a.C;
    float q = 0.0f;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        if (lane + 64 * u < V) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                f[u][i] -= mean;
                q = fmaf(f[u][i], f[u][i], q);
            }
        }
    }
    const float rstd = rsqrtf(wave_sum(q) / (float)a.C + a.eps);
    uint4* __restrict__ dst = (uint4*)((T*)a.y + (long)row * a.y_ld);
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int j = lane + 64 * u;
        if (j < V) {
#pragma unroll
            for (int i = 0; i < N; ++i) f[u][i] = fmaf(f[u][i] * rstd, gm[u][i], bt[u][i]);
            dst[j] = pack<T>(f[u]);
        }
    }
}

// y[r][c] = x[r][c] * gelu(x[r][C + c]), gelu(g) = g/2 * (1 + erf(g / sqrt 2)); one 16-byte
// output vector per thread.
template <typename T>
__global__ __launch_bounds__(256) void geglu_kernel(RowArgs a)
{
    constexpr int N = Vec16<T>::N;
    const int V = a.C / N;
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    const long row = e / V;
    if (row >= effective_rows(a)) return;
    const int j = (int)(e - row * V);
    const T* xr = (const T*)a.x + row * a.x_ld;
    float v[N], g[N];
    unpack<T>(*(const uint4*)(xr + j * N), v);
    unpack<T>(*(const uint4*)(xr + a.C + j * N), g);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] *= 0.5f * g[i] * (1.0f + erff(g[i] * 0.70710678118654752f));
    *(uint4*)((T*)a.y + row * a.y_ld + j * N) = pack<T>(v);
}

static int check_rows(const char* who, const void* x, const void* y, sige_dtype dt, int C, int x_ld, int y_ld,
                      int min_x_ld, const int32_t* count, int rows_per_count, int max_rows, int n_rows, int* launch)
{
    SIGE_REQUIRE(x && y, SIGE_ERR_INVALID_ARG, "%s: x and y are required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(C > 0 && x_ld >= min_x_ld && y_ld >= C, SIGE_ERR_INVALID_ARG, "%s: bad channel count or row stride", who);
    SIGE_REQUIRE(max_rows >= 0 && n_rows >= -1 && n_rows <= max_rows, n_rows > max_rows ? SIGE_ERR_CAPACITY : SIGE_ERR_INVALID_ARG,
                 "%s: need 0 <= n_rows <= max_rows (or n_rows = -1)", who);
    SIGE_REQUIRE(n_rows >= 0 || (count != nullptr && rows_per_count > 0), SIGE_ERR_INVALID_ARG,
                 "%s: count and rows_per_count are required when n_rows is -1", who);
    const size_t s = dtype_size(dt);
    SIGE_REQUIRE((C * s) % 16 == 0 && (x_ld * s) % 16 == 0 && (y_ld * s) % 16 == 0 && aligned16(x) && aligned16(y),
                 SIGE_ERR_UNSUPPORTED, "%s: C and the row strides must be multiples of %zu elements, pointers 16-byte aligned",
                 who, 16 / s);
    *launch = n_rows >= 0 ? n_rows : max_rows;
    return SIGE_OK;
}

template <typename T>
static int launch_norm(const RowArgs& a, int rows, hipStream_t st)
{
    const int V = a.C / Vec16<T>::N;
    const dim3 grid((rows + 3) / 4);
    if (V <= 64) hipLaunchKernelGGL((token_norm_kernel<T, 1>), grid, dim3(256), 0, st, a);
    else if (V <= 128) hipLaunchKernelGGL((token_norm_kernel<T, 2>), grid, dim3(256), 0, st, a);
    else if (V <= 256) hipLaunchKernelGGL((token_norm_kernel<T, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((token_norm_kernel<T, 8>), grid, dim3(256), 0, st, a);
    SIGE_LAUNCH_CHECK("sige_token_norm");
    return SIGE_OK;
}

}  // namespace sige

using namespace sige;

extern "C" int sige_token_norm(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, const int32_t* count,
                               int32_t rows_per_count, int32_t max_rows, int32_t n_rows, const float* gamma,
                               const float* beta, float eps, void* y, int32_t y_ld, void* stream)
{
    clear_error();
    const char* who = "sige_token_norm";
    int rows;
    if (int rc = check_rows(who, x, y, dt, C, x_ld, y_ld, C, count, rows_per_count, max_rows, n_rows, &rows)) return rc;
    SIGE_REQUIRE(C * dtype_size(dt) / 16 <= 512, SIGE_ERR_UNSUPPORTED, "%s: at most 8 KiB per token", who);
    if (rows == 0) return SIGE_OK;
    RowArgs a;
    a.x = x; a.y = y; a.gamma = gamma; a.beta = beta; a.count = count; a.C = C; a.x_ld = x_ld; a.y_ld = y_ld;
    a.rows_per_count = rows_per_count; a.max_rows = max_rows; a.n_host = n_rows; a.eps = eps;
    a.indices = nullptr; a.bh = a.bw = a.H = a.W = 0;
    a.d_pb = a.d_bw = fast_div(1);
    hipStream_t st = (hipStream_t)stream;
    return dt == SIGE_F32 ? launch_norm<float>(a, rows, st)
           : dt == SIGE_F16 ? launch_norm<f16>(a, rows, st) : launch_norm<bf16>(a, rows, st);
}

extern "C" int sige_gather_token_norm(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, const sige_geom* g,
                                      const int32_t* indices, const int32_t* count, int32_t max_blocks,
                                      int32_t n_blocks, const float* gamma, const float* beta, float eps,
                                      void* tiles, void* stream)
{
    clear_error();
    const char* who = "sige_gather_token_norm";
    int th, tw, nl;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(indices != nullptr, SIGE_ERR_INVALID_ARG, "%s: indices are required", who);
    SIGE_REQUIRE(g->k == 1 && g->stride == 1 && g->pad == 0, SIGE_ERR_UNSUPPORTED,
                 "%s: tokens are the pixels of the blocks themselves (k = 1, stride 1, no padding)", who);
    const long pb = (long)g->block_h * g->block_w;
    SIGE_REQUIRE(pb * max_blocks < (1L << 31), SIGE_ERR_UNSUPPORTED, "%s: too many tokens", who);
    int rows;
    if (int rc = check_rows(who, x, tiles, dt, C, x_ld, C, C, count, (int)pb, (int)(pb * max_blocks),
                            n_blocks >= 0 ? (int)(pb * n_blocks) : -1, &rows))
        return rc;
    SIGE_REQUIRE(C * dtype_size(dt) / 16 <= 512, SIGE_ERR_UNSUPPORTED, "%s: at most 8 KiB per token", who);
    if (rows == 0) return SIGE_OK;
    RowArgs a;
    a.x = x; a.y = tiles; a.gamma = gamma; a.beta = beta; a.count = count; a.C = C; a.x_ld = x_ld; a.y_ld = C;
    a.rows_per_count = (int)pb; a.max_rows = (int)(pb * max_blocks); a.n_host = n_blocks >= 0 ? (int)(pb * n_blocks) : -1;
    a.eps = eps;
    a.indices = indices; a.bh = g->block_h; a.bw = g->block_w; a.H = g->H_in; a.W = g->W_in;
    a.d_pb = fast_div(g->block_h * g->block_w);
    a.d_bw = fast_div(g->block_w);
    hipStream_t st = (hipStream_t)stream;
    return dt == SIGE_F32 ? launch_norm<float>(a, rows, st)
           : dt == SIGE_F16 ? launch_norm<f16>(a, rows, st) : launch_norm<bf16>(a, rows, st);
}

extern "C" int sige_geglu(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, const int32_t* count,
                          int32_t rows_per_count, int32_t max_rows, int32_t n_rows, void* y, int32_t y_ld,
                          void* stream)
{
    clear_error();
    const char* who = "sige_geglu";
    int rows;
    if (int rc = check_rows(who, x, y, dt, C, x_ld, y_ld, 2 * C, count, rows_per_count, max_rows, n_rows, &rows)) return rc;
    if (rows == 0) return SIGE_OK;
    RowArgs a;
    a.x = x; a.y = y; a.gamma = nullptr; a.beta = nullptr; a.count = count; a.C = C; a.x_ld = x_ld; a.y_ld = y_ld;
    a.rows_per_count = rows_per_count; a.max_rows = max_rows; a.n_host = n_rows; a.eps = 0.0f;
    a.indices = nullptr; a.bh = a.bw = a.H = a.W = 0;
    a.d_pb = a.d_bw = fast_div(1);
    const long n = (long)rows * (C * (long)dtype_size(dt) / 16);
    const long blocks = (n + 255) / 256;
    SIGE_REQUIRE(blocks < (1L << 31), SIGE_ERR_UNSUPPORTED, "%s: too many elements", who);
    hipStream_t st = (hipStream_t)stream;
    if (dt == SIGE_F32) hipLaunchKernelGGL((geglu_kernel<float>), dim3((int)blocks), dim3(256), 0, st, a);
    else if (dt == SIGE_F16) hipLaunchKernelGGL((geglu_kernel<f16>), dim3((int)blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((geglu_kernel<bf16>), dim3((int)blocks), dim3(256), 0, st, a);
    SIGE_LAUNCH_CHECK(who);
    return SIGE_OK;
}
