// sige_gather / sige_scatter (Fig. "method", Fig. "pipeline" (b)) with the cached-
// statistics Scale+Shift and the nonlinearity fused into the gather (Sec. 3.2
// "Pre-computing normalization parameters", "Kernel fusion").
//
// Both are pure HBM streams.  A tile row is one contiguous run of tile_w*C elements
// on either side, so every lane moves one 16-byte vector and a wave covers whole
// 1 KiB runs; the grid is (row groups) x (blocks), which keeps hundreds of
// workgroups in flight even when only a handful of blocks are active.
#include "common.h"

namespace sige {

struct GatherArgs {
    const void* x;
    void* tiles;
    const int32_t* indices;
    const int32_t* count;
    const float* scale;
    const float* shift;
    const void* mod;          // per-pixel modulation [Hin][Win][gamma C | beta C], or NULL
    int mod_ld_vec;
    int Hin, Win, ld_vec, V;  // V = 16-byte vectors per pixel, ld_vec = pixel stride in vectors
    int th, tw, stride, pad, up;
    int max_blocks, n_host, act, rows_per_wg;
    int segs, seg_px;   // few blocks: a tile row is cut into segs runs of seg_px pixels, one workgroup each
    int lv;             // log2(V) where V divides 256 (a power of two then): divisions by V are shifts
    FastDiv d_tw, d_segs;
};

// FIXED_CG: blockDim.x is a multiple of V, so a thread keeps one channel group and
// holds its scale/shift in registers.
template <typename T, bool FUSED, bool FIXED_CG>
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a)
{
    constexpr int N = Vec16<T>::N;
    const int n = blockIdx.y;
    int by0, bx0;
    if (n >= blocks_and_origin(a.count, a.max_blocks, a.n_host, a.indices, n, by0, bx0)) return;
    const int iy0 = by0 * a.stride - a.pad, ix0 = bx0 * a.stride - a.pad;
    int rg, seg;
    divmod(blockIdx.x, a.d_segs, rg, seg);
    const int r0 = rg * a.rows_per_wg;
    const int r1 = min(r0 + a.rows_per_wg, a.th);
    const int row_vecs = a.tw * a.V;
    const int total = (r1 - r0) * row_vecs;
    const uint4* __restrict__ src = (const uint4*)a.x;
    uint4* __restrict__ dst = (uint4*)a.tiles + ((long)n * a.th + r0) * row_vecs;
    const int Ws = a.Win >> a.up;

    float sc[N], sh[N];
    if (FUSED && FIXED_CG) {
        const int cg = threadIdx.x & (a.V - 1);
#pragma unroll
        for (int i = 0; i < N; ++i) { sc[i] = 1.0f; sh[i] = 0.0f; }
        if (a.scale != nullptr) {
            load_f32_run<N>(a.scale, cg * N, sc);
            load_f32_run<N>(a.shift, cg * N, sh);
        }
    }
    auto move = [&](int r, int px, int cg) {
        const int iy = iy0 + r0 + r, ix = ix0 + px;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (iy >= 0 && iy < a.Hin && ix >= 0 && ix < a.Win) {
            v = src[((long)(iy >> a.up) * Ws + (ix >> a.up)) * a.ld_vec + cg];
            if (FUSED) {
                float f[N];
                unpack<T>(v, f);
                if (!FIXED_CG) {
#pragma unroll
                    for (int i = 0; i < N; ++i) { sc[i] = 1.0f; sh[i] = 0.0f; }
                    if (a.scale != nullptr) {
                        load_f32_run<N>(a.scale, cg * N, sc);
                        load_f32_run<N>(a.shift, cg * N, sh);
                    }
                }
                if (a.mod == nullptr) {
                    scale_shift_act<N>(f, sc, sh, a.act);
                } else {
                    // spatially-adaptive: (scale * x + shift) * (1 + gamma) + beta, then the activation
                    const uint4* __restrict__ m = (const uint4*)a.mod + ((long)iy * a.Win + ix) * a.mod_ld_vec;
                    float gm[N], bt[N];
                    unpack<T>(m[cg], gm);
                    unpack<T>(m[a.V + cg], bt);
#pragma unroll
                    for (int i = 0; i < N; ++i) {
                        const float n = fmaf(sc[i], f[i], sh[i]);
                        f[i] = activate(fmaf(n, gm[i], n) + bt[i], a.act);
                    }
                }
                v = pack<T>(f);
            }
        }
        dst[(r * a.tw + px) * a.V + cg] = v;
    };
    if (a.segs > 1) {
        // one run of pixels of one tile row (rows_per_wg is 1 here)
        const int px0 = seg * a.seg_px, px1 = min(px0 + a.seg_px, a.tw);
        if (FIXED_CG) {
            const int ppi = 256 >> a.lv, cg = threadIdx.x & (a.V - 1);
            for (int px = px0 + (threadIdx.x >> a.lv); px < px1; px += ppi) move(0, px, cg);
        } else {
            for (int j = px0 * a.V + threadIdx.x; j < px1 * a.V; j += 256) {
                const int px = j / a.V;
                move(0, px, j - px * a.V);
            }
        }
    } else if (FIXED_CG) {
        // a thread keeps its channel group and walks over the pixels of the row group without
        // dividing: 256 / V pixels further each time
        const int ppi = 256 >> a.lv, cg = threadIdx.x & (a.V - 1);
        int step_r, step_x, r, px;
        divmod(ppi, a.d_tw, step_r, step_x);
        divmod(threadIdx.x >> a.lv, a.d_tw, r, px);
        const int nrows = r1 - r0;
        while (r < nrows) {
            move(r, px, cg);
            px += step_x;
            r += step_r;
            if (px >= a.tw) { px -= a.tw; ++r; }
        }
    } else {
        for (int j = threadIdx.x; j < total; j += 256) {
            const int r = j / row_vecs, jr = j - r * row_vecs;
            const int px = jr / a.V;
            move(r, px, jr - px * a.V);
        }
    }
}

struct ScatterArgs {
    const void* out_tiles;
    const void* res_tiles;
    const void* res_full;
    void* y;
    const int32_t* indices;
    const int32_t* count;
    int Hout, Wout, V, y_ld_vec, res_ld_vec;
    int bh, bw;
    int max_blocks, n_host, rows_per_wg;
    int lv;             // log2(V) where V divides 256
    FastDiv d_bw;       // for blocks that are not clipped at the right edge (cols == bw)
};

template <typename T, bool ADD>
__global__ __launch_bounds__(256) void scatter_kernel(ScatterArgs a)
{
    constexpr int N = Vec16<T>::N;
    const int n = blockIdx.y;
    int y0, x0;
    if (n >= blocks_and_origin(a.count, a.max_blocks, a.n_host, a.indices, n, y0, x0)) return;
    if (y0 < 0 || x0 < 0 || y0 >= a.Hout || x0 >= a.Wout) return;  // never store outside y
    const int r0 = blockIdx.x * a.rows_per_wg;
    const int r1 = min(min(r0 + a.rows_per_wg, a.bh), a.Hout - y0);  // clip rows at the bottom edge
    if (r1 <= r0) return;
    const int cols = min(a.bw, a.Wout - x0);                         // clip columns at the right edge
    const int row_vecs = cols * a.V;
    const int total = (r1 - r0) * row_vecs;
    const uint4* __restrict__ src = (const uint4*)a.out_tiles;
    const uint4* __restrict__ rt = (const uint4*)a.res_tiles;
    const uint4* __restrict__ rf = (const uint4*)a.res_full;
    uint4* __restrict__ dst = (uint4*)a.y;
    auto move = [&](int r, int px, int cg) {
        const long t = (((long)n * a.bh + r0 + r) * a.bw + px) * a.V + cg;
        const long pix = (long)(y0 + r0 + r) * a.Wout + x0 + px;
        uint4 v = src[t];
        if (ADD) {
            float f[N], g[N];
            unpack<T>(v, f);
            if (rt) {
                unpack<T>(rt[t], g);
#pragma unroll
                for (int i = 0; i < N; ++i) f[i] += g[i];
            }
            if (rf) {
                unpack<T>(rf[pix * a.res_ld_vec + cg], g);
#pragma unroll
                for (int i = 0; i < N; ++i) f[i] += g[i];
            }
            v = pack<T>(f);
        }
        dst[pix * a.y_ld_vec + cg] = v;
    };
    if (256 % a.V == 0) {
        // division-free walk: a thread keeps its channel group, 256 / V pixels further each time;
        // the tile vectors (and residuals) of U pixels are loaded before any is stored
        constexpr int U = 4;
        const int ppi = 256 >> a.lv, cg = threadIdx.x & (a.V - 1);
        const int p = threadIdx.x >> a.lv;
        int step_r, step_x, r, px;
        if (cols == a.bw) {              // the usual case: divisor known on the host
            divmod(ppi, a.d_bw, step_r, step_x);
            divmod(p, a.d_bw, r, px);
        } else {
            step_r = ppi / cols; step_x = ppi - step_r * cols;
            r = p / cols; px = p - r * cols;
        }
        const int nrows = r1 - r0;
        while (r < nrows) {
            uint4 v[U], q1[U], q2[U];
            long pix[U];
            bool in[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                in[u] = r < nrows;
                const int rr = in[u] ? r : 0, pp = in[u] ? px : 0;     // a valid element when past the end
                const long t = (((long)n * a.bh + r0 + rr) * a.bw + pp) * a.V + cg;
                pix[u] = (long)(y0 + r0 + rr) * a.Wout + x0 + pp;
                v[u] = src[t];
                if (ADD) {
                    if (rt) q1[u] = rt[t];
                    if (rf) q2[u] = rf[pix[u] * a.res_ld_vec + cg];
                }
                px += step_x;
                r += step_r;
                if (px >= cols) { px -= cols; ++r; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!in[u]) break;
                uint4 w = v[u];
                if (ADD) {
                    float f[N], g[N];
                    unpack<T>(w, f);
                    if (rt) {
                        unpack<T>(q1[u], g);
#pragma unroll
                        for (int i = 0; i < N; ++i) f[i] += g[i];
                    }
                    if (rf) {
                        unpack<T>(q2[u], g);
#pragma unroll
                        for (int i = 0; i < N; ++i) f[i] += g[i];
                    }
                    w = pack<T>(f);
                }
                dst[pix[u] * a.y_ld_vec + cg] = w;
            }
        }
    } else {
        for (int j = threadIdx.x; j < total; j += 256) {
            const int r = j / row_vecs, jr = j - r * row_vecs;
            const int px = jr / a.V;
            move(r, px, jr - px * a.V);
        }
    }
}

// Rows per workgroup: about `target` bytes each (measured on a 512 MB tensor: plain copies run
// fastest with ~8 KiB per workgroup, two vectors per lane; the fused gather needs ~40 KiB to
// amortise the scale/shift each lane fetches first), but at least ~2048 workgroups in total.
static int pick_rows(int rows, size_t row_bytes, int blocks, size_t target)
{
    int rpw = (int)((target + row_bytes - 1) / row_bytes);
    if (rpw < 1) rpw = 1;
    while (rpw > 1 && (long)blocks * ((rows + rpw - 1) / rpw) < 2048) --rpw;
    return rpw > rows ? rows : rpw;
}

template <typename T>
static void launch_gather(const GatherArgs& a, dim3 grid, bool fused, hipStream_t st)
{
    // the fixed-channel-group walk needs a whole number of pixels per 256 threads (V > 256 would
    // never advance)
    const bool fixed = (256 % a.V) == 0;
    if (!fused && fixed)
        hipLaunchKernelGGL((gather_kernel<T, false, true>), grid, dim3(256), 0, st, a);
    else if (!fused)
        hipLaunchKernelGGL((gather_kernel<T, false, false>), grid, dim3(256), 0, st, a);
    else if (fixed)
        hipLaunchKernelGGL((gather_kernel<T, true, true>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((gather_kernel<T, true, false>), grid, dim3(256), 0, st, a);
}

template <typename T>
static void launch_scatter(const ScatterArgs& a, dim3 grid, hipStream_t st)
{
    if (a.res_tiles || a.res_full)
        hipLaunchKernelGGL((scatter_kernel<T, true>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((scatter_kernel<T, false>), grid, dim3(256), 0, st, a);
}

}  // namespace sige

using namespace sige;

static int run_gather(const char* who, const void* x, sige_dtype dt, int32_t C, int32_t x_ld, int32_t up,
                      const sige_geom* g, const int32_t* indices, const int32_t* count,
                      int32_t max_blocks, int32_t n_blocks, const float* scale, const float* shift,
                      const void* mod, int32_t mod_ld, sige_act act, void* tiles, void* stream)
{
    int th, tw, nl;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(x && indices && tiles, SIGE_ERR_INVALID_ARG, "%s: x, indices and tiles are required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(C > 0 && x_ld >= C, SIGE_ERR_INVALID_ARG, "%s: need C > 0 and x_ld >= C", who);
    SIGE_REQUIRE((scale == nullptr) == (shift == nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: scale and shift must be given together", who);
    SIGE_REQUIRE(act_ok((int)act), SIGE_ERR_INVALID_ARG, "%s: unknown activation %d", who, (int)act);
    SIGE_REQUIRE(up == 0 || up == 1, SIGE_ERR_INVALID_ARG, "%s: up must be 0 or 1", who);
    SIGE_REQUIRE(up == 0 || (g->H_in % 2 == 0 && g->W_in % 2 == 0), SIGE_ERR_INVALID_ARG,
                 "%s: up-sampled input size must be even", who);
    const size_t s = dtype_size(dt);
    SIGE_REQUIRE((C * s) % 16 == 0 && (x_ld * s) % 16 == 0, SIGE_ERR_UNSUPPORTED,
                 "%s: C and x_ld must be multiples of %zu elements (16 bytes)", who, 16 / s);
    SIGE_REQUIRE(aligned16(x) && aligned16(tiles), SIGE_ERR_UNSUPPORTED, "%s: pointers must be 16-byte aligned", who);
    if (nl == 0) return SIGE_OK;
    GatherArgs a;
    a.x = x; a.tiles = tiles; a.indices = indices; a.count = count; a.scale = scale; a.shift = shift;
    a.Hin = g->H_in; a.Win = g->W_in; a.V = (int)(C * s / 16); a.ld_vec = (int)(x_ld * s / 16);
    a.th = th; a.tw = tw; a.stride = g->stride; a.pad = g->pad; a.up = up;
    a.max_blocks = max_blocks; a.n_host = n_blocks; a.act = (int)act;
    a.mod = mod; a.mod_ld_vec = (int)(mod_ld * s / 16);
    if (mod != nullptr)
        SIGE_REQUIRE(mod_ld >= 2 * C && (mod_ld * s) % 16 == 0 && aligned16(mod), SIGE_ERR_UNSUPPORTED,
                     "%s: mod must be 16-byte aligned with a pixel stride >= 2C that is a multiple of %zu elements",
                     who, 16 / s);
    const bool fused = scale != nullptr || act != SIGE_ACT_NONE || mod != nullptr;
    a.rows_per_wg = pick_rows(th, (size_t)tw * C * s, nl, fused ? 40960 : 8192);
    // Few blocks: even one tile row per workgroup leaves most of the chip idle and every thread
    // with a chain of dependent iterations.  The rows are cut into runs of pixels, down to one
    // iteration of the 256 threads per workgroup, until about 1024 workgroups exist.
    a.segs = 1;
    a.seg_px = tw;
    if (a.rows_per_wg == 1 && (long)nl * th < 1024) {
        const int V = (int)((size_t)C * s / 16);
        const int min_px = std::max(1, 256 / std::max(V, 1));          // pixels of one iteration
        const int want = (int)((1024 + (long)nl * th - 1) / ((long)nl * th));
        const int seg_px = std::max(min_px, (tw + want - 1) / want);
        a.seg_px = seg_px;
        a.segs = (tw + seg_px - 1) / seg_px;
    }
    a.lv = 0;
    while ((1 << (a.lv + 1)) <= a.V && a.lv < 8) ++a.lv;      // floor(log2 V); exact where V divides 256
    a.d_tw = fast_div(tw);
    a.d_segs = fast_div(a.segs);
    dim3 grid(((th + a.rows_per_wg - 1) / a.rows_per_wg) * a.segs, nl);
    SIGE_REQUIRE(nl <= 65535, SIGE_ERR_UNSUPPORTED, "%s: more than 65535 blocks per launch", who);
    hipStream_t st = (hipStream_t)stream;
    if (dt == SIGE_F32) launch_gather<float>(a, grid, fused, st);
    else if (dt == SIGE_F16) launch_gather<f16>(a, grid, fused, st);
    else launch_gather<bf16>(a, grid, fused, st);
    SIGE_LAUNCH_CHECK(who);
    return SIGE_OK;
}

extern "C" int sige_gather(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, int32_t up,
                           const sige_geom* g, const int32_t* indices, const int32_t* count,
                           int32_t max_blocks, int32_t n_blocks, const float* scale,
                           const float* shift, sige_act act, void* tiles, void* stream)
{
    clear_error();
    return run_gather("sige_gather", x, dt, C, x_ld, up, g, indices, count, max_blocks, n_blocks, scale, shift,
                      nullptr, 0, act, tiles, stream);
}

extern "C" int sige_gather_modulated(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, int32_t up,
                                     const sige_geom* g, const int32_t* indices, const int32_t* count,
                                     int32_t max_blocks, int32_t n_blocks, const float* scale,
                                     const float* shift, const void* mod, int32_t mod_ld, sige_act act,
                                     void* tiles, void* stream)
{
    clear_error();
    SIGE_REQUIRE(mod != nullptr, SIGE_ERR_INVALID_ARG, "sige_gather_modulated: mod is required");
    return run_gather("sige_gather_modulated", x, dt, C, x_ld, up, g, indices, count, max_blocks, n_blocks, scale,
                      shift, mod, mod_ld, act, tiles, stream);
}

extern "C" int sige_scatter(const void* out_tiles, sige_dtype dt, const sige_geom* g, int32_t Cout,
                            const int32_t* indices, const int32_t* count, int32_t max_blocks,
                            int32_t n_blocks, const void* residual_tiles, const void* residual,
                            int32_t res_ld, void* y, int32_t y_ld, void* stream)
{
    clear_error();
    const char* who = "sige_scatter";
    int nl;
    if (int rc = check_geom(g, who, nullptr, nullptr)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(out_tiles && indices && y, SIGE_ERR_INVALID_ARG, "%s: out_tiles, indices and y are required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cout > 0 && y_ld >= Cout, SIGE_ERR_INVALID_ARG, "%s: need Cout > 0 and y_ld >= Cout", who);
    SIGE_REQUIRE(residual == nullptr || res_ld >= Cout, SIGE_ERR_INVALID_ARG, "%s: res_ld must be >= Cout", who);
    const size_t s = dtype_size(dt);
    SIGE_REQUIRE((Cout * s) % 16 == 0 && (y_ld * s) % 16 == 0 && (residual == nullptr || (res_ld * s) % 16 == 0),
                 SIGE_ERR_UNSUPPORTED, "%s: Cout and pixel strides must be multiples of %zu elements (16 bytes)",
                 who, 16 / s);
    SIGE_REQUIRE(aligned16(out_tiles) && aligned16(y) && aligned16(residual_tiles) && aligned16(residual),
                 SIGE_ERR_UNSUPPORTED, "%s: pointers must be 16-byte aligned", who);
    SIGE_REQUIRE(nl <= 65535, SIGE_ERR_UNSUPPORTED, "%s: more than 65535 blocks per launch", who);
    if (nl == 0) return SIGE_OK;
    ScatterArgs a;
    a.out_tiles = out_tiles; a.res_tiles = residual_tiles; a.res_full = residual; a.y = y;
    a.indices = indices; a.count = count;
    a.Hout = g->H_out; a.Wout = g->W_out; a.V = (int)(Cout * s / 16);
    a.y_ld_vec = (int)(y_ld * s / 16); a.res_ld_vec = residual ? (int)(res_ld * s / 16) : 0;
    a.bh = g->block_h; a.bw = g->block_w;
    a.max_blocks = max_blocks; a.n_host = n_blocks;
    a.rows_per_wg = pick_rows(g->block_h, (size_t)g->block_w * Cout * s, nl, 8192);
    a.lv = 0;
    while ((1 << (a.lv + 1)) <= a.V && a.lv < 8) ++a.lv;
    a.d_bw = fast_div(g->block_w);
    dim3 grid((g->block_h + a.rows_per_wg - 1) / a.rows_per_wg, nl);
    hipStream_t st = (hipStream_t)stream;
    if (dt == SIGE_F32) launch_scatter<float>(a, grid, st);
    else if (dt == SIGE_F16) launch_scatter<f16>(a, grid, st);
    else launch_scatter<bf16>(a, grid, st);
    SIGE_LAUNCH_CHECK(who);
    return SIGE_OK;
}
