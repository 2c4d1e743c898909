// sige_conv: the convolution F_l on the stacked active tiles (Fig. "method"), with bias
// (Fig. "pipeline" (b)), as an implicit GEMM on the gfx950 matrix cores:
//     M = pixels of the active blocks, N = Cout, K = k*k*Cin.
//
// A workgroup (4 waves) owns an M x N patch: a row band of one block (or several
// whole small blocks) times a slab of output channels.  The input rows it needs
// (band + halo) are staged once per channel chunk into LDS and reused by all k*k
// taps; the A operand of each MFMA is a 16-byte LDS read at
// pixel(py*stride+ky, px*stride+kx), the B operand a 16-byte read of weights that
// sige_pack_weight has laid out in fragment order (L2 resident, shared by every
// workgroup), prefetched through a register ring.  fp32 accumulation, bias added when
// the accumulators leave the registers, one rounding to the storage type at the store.
// sige_fused_conv is the same kernel with the gather folded into the staging and the
// scatter into the epilogue (sige_conv_scatter: the scatter only); with a workspace, calls
// with few workgroups and a long K are cut along K and finished by conv_reduce_kernel, or
// - without staged arithmetic and up to two chunks - take a shape whose four or eight waves split K
// with the whole of Cin (or half) staged at once.  1x1 calls with few rows have a kernel of their
// own further down (pointwise_kernel); two independent fused calls can share one launch
// (conv_pair_kernel, sige_fused_conv_pair).
// The epilogue can also write activated copies of the output for the layers that
// normalise it next (Sec. 3.2 "Pre-computing normalization parameters": their Scale+Shift
// is a constant per channel).
//
// This file holds the planning and the entry points; the kernels live in conv_kernels.h and are
// instantiated once per storage type in conv_f32.hip, conv_f16.hip and conv_bf16.hip.
#include "conv_kernels.h"

namespace sige {

// instantiated in conv_f32.hip, conv_f16.hip and conv_bf16.hip
SIGE_CONV_LAUNCHERS(extern, float)
SIGE_CONV_LAUNCHERS(extern, f16)
SIGE_CONV_LAUNCHERS(extern, bf16)

// Chooses the workgroup shape and the staged channel chunk for one call, then - when the caller
// gave a workspace (partial_elems = fp32 elements it holds) and the call has few workgroups but a
// long K - how many workgroups share one output patch along K.
static bool plan_conv(const sige_geom* g, int th, int tw, int Cin, int Cout, size_t s, int kstep,
                      int nblocks, size_t partial_elems, bool staged_math, ConvPlan* best)
{
    // overrides for tests and tuning runs (sige_set_knob; -1 = automatic): the shape / the K steps per chunk
    const int force_cfg = knob(SIGE_KNOB_CONV_CFG), force_kc_v = knob(SIGE_KNOB_CONV_KC);
    const bool force = force_cfg >= 0, force_kc = force_kc_v >= 0;
    const bool force_whole = force && force_cfg >= 3 && force_kc && force_kc_v >= 16;
    double best_score = -1.0;
    // bytes between the staged pixels' channel runs: 48 behind runs of up to 256 bytes (measured 3 - 5 % faster
    // than 16 with every block active: 902 vs 874 TFLOP/s at 1024 x 1024 x 128, 1014 vs 987 at 512 x 512 x 256),
    // 16 behind the long runs of the shapes that stage the whole of Cin, which have no LDS to spare
    auto pad_of = [&](int kc) {
        const int k = knob(SIGE_KNOB_CONV_LDS_PAD);
        return k > 0 ? k : (kc * kstep * (int)s <= 256 ? 48 : 16);
    };
    auto lds_bytes = [&](int cfg, long npix, int kc) {
        size_t lds = (size_t)npix * (kc * kstep * s + pad_of(kc));
        return std::max(lds, (size_t)kCfg[cfg].WK * kCfg[cfg].M * (kCfg[cfg].N + 4) * sizeof(float));   // the epilogue's staging
    };
    // a compute unit has 160 KiB of LDS: one workgroup where a single chunk is all there is to overlap,
    // two otherwise; the kernel's own static array (the block origins) counts too
    constexpr size_t kStaticLds = 2 * MAX_G * sizeof(int);
    auto lds_fits = [&](int cfg, size_t lds, int kc) {
        return lds + kStaticLds <= (kc == 1 || (kc == 4 && kCfg[cfg].WK == 4) ? 160u : 80u) * 1024u;
    };
    for (int cfg = 0; cfg < kNumCfg; ++cfg) {
        if (force && !force_whole && force_cfg != cfg) continue;
        if (g->k != 1 && g->k != 3 && cfg != 2) continue;   // only the plain 64x64 shape is built for other k
        const int M = kCfg[cfg].M, Nn = kCfg[cfg].N, WK = kCfg[cfg].WK;
        if (g->block_w > M) continue;
        ConvPlan p;
        p.cfg = cfg;
        p.ksplit = 1;
        const int pbfull = g->block_h * g->block_w;
        if (pbfull <= M) { p.G = M / pbfull; p.rows = g->block_h; }
        else { p.G = 1; p.rows = M / g->block_w; }
        p.bands = (g->block_h + p.rows - 1) / p.rows;
        p.trows = (p.rows - 1) * g->stride + g->k;
        p.slabs = (Cout + Nn - 1) / Nn;
        p.groups = (nblocks + p.G - 1) / p.G;
        const long npix = (long)p.G * p.trows * tw;
        // K steps per chunk: the largest of 8 / 4 / 3 / 1 that divides Cin and whose staged tile fits
        // (3: the 48 channels of a label-map convolution in one chunk)
        p.kc = 0;
        for (int kc : {8, 4, 3, 1}) {
            if (force_kc && !force_whole && force_kc_v != kc) continue;
            if (kc % WK || Cin % (kc * kstep)) continue;
            if (g->k != 1 && g->k != 3 && kc != 1) continue;
            const size_t lds = lds_bytes(cfg, npix, kc);
            if (lds_fits(cfg, lds, kc)) { p.kc = kc; p.lds = lds; break; }
        }
        if (p.kc == 0) continue;
        p.Cc = p.kc * kstep;
        p.ps = (int)(p.Cc * s + pad_of(p.kc));
        const double util = (double)(p.G > 1 ? std::min(p.G, nblocks) * pbfull
                                             : std::min(p.rows, (int)g->block_h) * g->block_w) / M;
        const long wgs = (long)p.groups * p.bands * p.slabs;
        const double fill = wgs >= 512 ? 1.0 : (double)wgs / 512.0;
        const double bonus = cfg == 0 ? 1.0 : cfg == 1 ? 0.9 : cfg == 2 ? 0.75 : 0.7;
        const double nuse = (double)Cout / (p.slabs * Nn);
        const double score = util * fill * bonus * nuse;
        if (score > best_score) { best_score = score; *best = p; }
    }
    if (best_score < 0.0) return false;
    // K split over workgroups.  A workgroup walks through its channel chunks one after the other and
    // each costs a staging round trip (a few microseconds), so a call with at most one workgroup per
    // compute unit and at least three chunks (320 channels or more in the half types) is cut along K,
    // to about 200 workgroups in all: measured with weights that come from HBM (a network's do), more
    // shares than that cost more in the second kernel than they save in the first.  Smaller chunks
    // when that is what it takes to reach 256 workgroups.
    ConvPlan& p = *best;
    const int force_split_v = knob(SIGE_KNOB_CONV_SPLIT);
    const bool force_split = force_split_v >= 0;
    // Few workgroups and a long K, nothing to compute while staging (no Scale+Shift, no activation):
    // 64 x 32 patches whose waves split K, with the whole of Cin (or half of it) staged at once -
    // eight waves over 256, 512 or 640 channels, four over 320.  One kernel, no workspace; the waves'
    // sums meet in LDS.  (With staged arithmetic the chunk would cost every workgroup many times the
    // activation work of the plain four-wave shape's.)
    if (g->k == 3 && g->block_w <= 64 &&
        (force_whole || (!staged_math && !force && !force_kc && !force_split && Cin >= 20 * kstep))) {
        ConvPlan q;
        q.ksplit = 1;
        const int M = 64, pbfull = g->block_h * g->block_w;
        if (pbfull <= M) { q.G = M / pbfull; q.rows = g->block_h; }
        else { q.G = 1; q.rows = M / g->block_w; }
        q.bands = (g->block_h + q.rows - 1) / q.rows;
        q.trows = (q.rows - 1) * g->stride + g->k;
        q.slabs = (Cout + 31) / 32;
        q.groups = (nblocks + q.G - 1) / q.G;
        const long npix = (long)q.G * q.trows * tw;
        q.kc = 0;
        static const int cand[4][2] = {{4, 40}, {4, 32}, {4, 16}, {3, 20}};   // shape, K steps per chunk
        for (const auto& c : cand) {
            if (force_whole && (force_cfg != c[0] || force_kc_v != c[1])) continue;
            // at most two chunks: beyond that a workgroup streams so much weight by itself that the
            // cut over workgroups below, second kernel included, is faster
            if (Cin % (c[1] * kstep) || (!force_whole && Cin / (c[1] * kstep) > (c[1] == 40 ? 1 : 2))) continue;
            const size_t lds = lds_bytes(c[0], npix, c[1]);
            if (lds <= (c[0] == 4 ? 150u : 75u) * 1024u) { q.cfg = c[0]; q.kc = c[1]; q.lds = lds; break; }
        }
        long wgs4 = (long)q.groups * q.bands * q.slabs;
        // at most 64 workgroups (a 512-channel layer at 8 x 8 has 16): patches of 32 rows instead of
        // 64, so that twice as many compute units stream the weight and share the MFMAs
        const int half_knob = knob(SIGE_KNOB_CONV_HALF);     // most workgroups for which rows are halved
        const long half_max = half_knob >= 0 ? half_knob : 64;
        if (q.kc && q.cfg == 4 && wgs4 <= half_max && pbfull >= 64 && g->block_w <= 32) {
            q.cfg = 5;
            q.G = 1;
            q.rows = 32 / g->block_w;
            q.bands = (g->block_h + q.rows - 1) / q.rows;
            q.trows = (q.rows - 1) * g->stride + g->k;
            q.groups = nblocks;
            q.lds = lds_bytes(5, (long)q.trows * tw, q.kc);
            wgs4 = (long)q.groups * q.bands * q.slabs;
        }
        if (q.kc && (wgs4 <= 256 || force_whole)) {
            q.Cc = q.kc * kstep;
            q.ps = (int)(q.Cc * s + pad_of(q.kc));
            p = q;
            if (!force_whole) return true;
        }
    }
    const long wgs = (long)p.groups * p.bands * p.slabs;
    const size_t per_split = (size_t)nblocks * g->block_h * g->block_w * Cout;
    const int max_by_ws = per_split ? (int)std::min<size_t>(partial_elems / per_split, 64) : 0;
    if (max_by_ws >= 2 && (g->k == 1 || g->k == 3) && p.kc >= 4) {
        const int WK = kCfg[p.cfg].WK;
        int kc = p.kc;
        if (kc == 8 && wgs * (Cin / (8 * kstep)) < 256 && 4 % WK == 0 && !force_kc) kc = 4;
        const int nch = Cin / (kc * kstep);
        int S = 1;
        const int tw_knob = knob(SIGE_KNOB_CONV_SPLIT_WGS);
        const long target = tw_knob >= 0 ? tw_knob : 200;
        if (wgs <= 256 && nch >= 3 && Cin >= 20 * kstep) S = (int)std::min<long>(nch, (target + wgs - 1) / wgs);
        if (force_split) S = std::min(force_split_v, nch);
        S = std::max(1, std::min(S, max_by_ws));
        if (S > 1) {
            if (kc != p.kc) {
                const long npix = (long)p.G * p.trows * tw;
                p.kc = kc;
                p.lds = lds_bytes(p.cfg, npix, kc);
                p.Cc = kc * kstep;
                p.ps = (int)(p.Cc * s + pad_of(p.kc));
            }
            p.ksplit = S;
        }
    }
    return true;
}

}  // namespace sige

using namespace sige;

extern "C" size_t sige_packed_weight_bytes(sige_dtype dt, int32_t Cout, int32_t Cin, int32_t k)
{
    if (!dtype_ok(dt) || Cout <= 0 || Cin <= 0 || k <= 0) return 0;
    const int ks = dt == SIGE_F32 ? 8 : 16;
    if (Cin % ks) return 0;
    return (size_t)((Cout + 31) / 32) * k * k * (Cin / ks) * 64 * 16;
}

extern "C" int sige_pack_weight(const void* w_oihw, sige_dtype dt, int32_t Cout, int32_t Cin, int32_t k,
                                void* packed, void* stream)
{
    clear_error();
    const char* who = "sige_pack_weight";
    SIGE_REQUIRE(w_oihw && packed, SIGE_ERR_INVALID_ARG, "%s: NULL pointer", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cout > 0 && Cin > 0 && k > 0 && (k & 1), SIGE_ERR_INVALID_ARG, "%s: bad shape", who);
    const int ks = dt == SIGE_F32 ? 8 : 16;
    SIGE_REQUIRE(Cin % ks == 0, SIGE_ERR_UNSUPPORTED, "%s: Cin must be a multiple of %d for this dtype", who, ks);
    const size_t bytes = sige_packed_weight_bytes(dt, Cout, Cin, k);
    const long n = (long)(bytes / dtype_size(dt));
    const long blocks = (n + 255) / 256;
    SIGE_REQUIRE(blocks < (1L << 31), SIGE_ERR_UNSUPPORTED, "%s: weight too large", who);
    hipStream_t st = (hipStream_t)stream;
    return dt == SIGE_F32   ? launch_pack<float>(w_oihw, Cout, Cin, k, n, packed, st)
           : dt == SIGE_F16 ? launch_pack<f16>(w_oihw, Cout, Cin, k, n, packed, st)
                            : launch_pack<bf16>(w_oihw, Cout, Cin, k, n, packed, st);
}

// Whether a call goes to pointwise_kernel, and with which patch per workgroup (0 = not; 1: 64 rows
// x 32 channels, 2: 64 x 64, 3: 32 x 32 where the larger patches would leave most compute units
// without work): a plain 1x1 (no scale, shift or activation on the way in), an even number of
// K steps, and few enough rows that its patches do not fill the compute units more than once (then
// the tiled kernel, which reads every weight once per 128 rows, is the better one).
static int pointwise_tiles(const sige_geom* g, const ConvArgs& a, int ks, int nl)
{
    const int force_v = knob(SIGE_KNOB_CONV_POINTWISE);     // 0 = never, 1 / 2 / 3 = that patch
    const bool force = force_v >= 0;
    if (force && force_v == 0) return 0;
    if (g->k != 1 || g->stride != 1 || g->pad != 0 || a.up != 0 || a.scale != nullptr || a.act != SIGE_ACT_NONE)
        return 0;
    const int kcs = a.Cin / ks;
    if (kcs % 2 || (kcs < 20 && !force)) return 0;          // a short K is the tiled kernel's (one staged chunk)
    const long rows = (long)nl * g->block_h * g->block_w;
    const long mt = (rows + 63) / 64, nt = (a.Cout + 31) / 32;
    if ((rows + 31) / 32 > 65535) return 0;
    if (force) return std::min(std::max(force_v, 1), 3);
    // the smallest patch that still fits one workgroup per compute unit
    if ((rows + 31) / 32 * nt <= 256) return 3;
    if (mt * nt <= 256) return 1;
    if (mt * ((nt + 1) / 2) <= (kcs >= 64 ? 512 : 256)) return 2;   // a long K: better two rounds here than the tiled kernel's chunks
    return 0;
}

// Shared by sige_conv, sige_conv_scatter and sige_fused_conv: plan and fill the arguments ...
static int prepare_conv(const char* who, sige_dtype dt, const sige_geom* g, int th, int tw, int Cin, int Cout,
                        int max_blocks, int n_blocks, int nl, ConvArgs& a, void* workspace, size_t workspace_bytes,
                        ConvPlan* p, int* pointwise)
{
    const int ks = dt == SIGE_F32 ? 8 : 16;
    a.bh = g->block_h; a.bw = g->block_w; a.Cin = Cin; a.Cout = Cout; a.max_blocks = max_blocks; a.n_host = n_blocks;
    a.d_bw = fast_div(g->block_w);
    a.d_pbfull = fast_div(g->block_h * g->block_w);
    a.d_runs = fast_div((Cout + (int)(16 / dtype_size(dt)) - 1) / (int)(16 / dtype_size(dt)));
    *pointwise = pointwise_tiles(g, a, ks, nl);
    if (*pointwise) return SIGE_OK;
    const bool ws_ok = workspace != nullptr && (reinterpret_cast<uintptr_t>(workspace) & 15u) == 0;
    SIGE_REQUIRE(plan_conv(g, th, tw, Cin, Cout, dtype_size(dt), ks, nl, ws_ok && !a.glu ? workspace_bytes / sizeof(float) : 0,
                           a.scale != nullptr || a.act != SIGE_ACT_NONE, p),
                 SIGE_ERR_UNSUPPORTED, "%s: no kernel shape fits block %dx%d, k %d, stride %d, Cin %d", who,
                 g->block_h, g->block_w, g->k, g->stride, Cin);
    SIGE_REQUIRE(p->groups <= 65535 && p->bands * p->ksplit <= 65535, SIGE_ERR_UNSUPPORTED,
                 "%s: too many blocks per launch", who);
    a.th = th; a.tw = tw; a.bh = g->block_h; a.bw = g->block_w; a.k = g->k; a.stride = g->stride;
    a.Cin = Cin; a.Cout = Cout; a.max_blocks = max_blocks; a.n_host = n_blocks;
    a.G = p->G; a.rows = p->rows; a.trows = p->trows; a.Cc = p->Cc; a.ps = p->ps;
    a.bands = p->bands; a.ksplit = p->ksplit;
    a.d_bands = fast_div(p->bands); a.d_ksplit = fast_div(p->ksplit); a.d_mk_nbx = fast_div(1);
    a.direct = knob(SIGE_KNOB_CONV_DIRECT) != 0;
    // 128 x 128 shape with at least two rounds of workgroups: every other workgroup of the first round starts one
    // sleep unit (3 us) late, so that the two workgroups of a compute unit do not stage, multiply and store in
    // step (measured + 2 - 4 % at 512 x 512 and 1024 x 1024 with 128 channels; with a single round it only costs,
    // and so it does on a 1x1 call, whose two rounds are memory traffic from start to end: 30 -> 32.5 us)
    a.stagger = (p->cfg == 0 && g->k >= 3 && (long)p->groups * p->bands * p->slabs * p->ksplit >= 1024) ? 1 : 0;
    a.d_pb = fast_div(p->rows * g->block_w);
    a.d_per = fast_div(p->trows * tw);
    a.d_tw = fast_div(tw);
    a.partial = p->ksplit > 1 ? (float*)workspace : nullptr;
    a.partial_stride = (long)nl * g->block_h * g->block_w * Cout;
    return SIGE_OK;
}

// ... and launch.
static int launch_prepared(sige_dtype dt, const ConvArgs& a, const ConvPlan& p, int pointwise, int nl, hipStream_t st)
{
    if (pointwise)
        return dt == SIGE_F32 ? launch_pointwise<float>(a, nl, pointwise, st)
               : dt == SIGE_F16 ? launch_pointwise<f16>(a, nl, pointwise, st) : launch_pointwise<bf16>(a, nl, pointwise, st);
    int rc = dt == SIGE_F32 ? launch_conv<float>(a, p, st)
             : dt == SIGE_F16 ? launch_conv<f16>(a, p, st) : launch_conv<bf16>(a, p, st);
    if (rc || p.ksplit == 1) return rc;
    return dt == SIGE_F32 ? launch_reduce<float>(a, nl, st)
           : dt == SIGE_F16 ? launch_reduce<f16>(a, nl, st) : launch_reduce<bf16>(a, nl, st);
}

static int run_conv(const char* who, sige_dtype dt, const sige_geom* g, int th, int tw, int Cin, int Cout,
                    int max_blocks, int n_blocks, int nl, ConvArgs& a, void* workspace, size_t workspace_bytes,
                    void* stream)
{
    ConvPlan p;
    int pointwise = 0;
    if (int rc = prepare_conv(who, dt, g, th, tw, Cin, Cout, max_blocks, n_blocks, nl, a, workspace, workspace_bytes,
                              &p, &pointwise))
        return rc;
    return launch_prepared(dt, a, p, pointwise, nl, (hipStream_t)stream);
}

extern "C" size_t sige_conv_workspace_bytes(sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                                            int32_t max_blocks)
{
    int th, tw;
    if (!dtype_ok(dt) || Cin <= 0 || Cout <= 0 || max_blocks <= 0 || check_geom(g, "sige_conv_workspace_bytes", &th, &tw))
        return 0;
    const int ks = dt == SIGE_F32 ? 8 : 16;
    if (Cin % ks) return 0;
    size_t need = 0;
    for (int nl = 1; nl <= max_blocks; ++nl) {
        ConvPlan p;
        if (!plan_conv(g, th, tw, Cin, Cout, dtype_size(dt), ks, nl, (size_t)1 << 40, true, &p)) return 0;
        if (p.ksplit > 1) need = std::max(need, (size_t)p.ksplit * nl * g->block_h * g->block_w * Cout * sizeof(float));
        else if ((long)p.groups * p.bands * p.slabs > 256) break;   // more blocks only add workgroups
    }
    return need;
}

extern "C" int sige_conv_plan(sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout, int32_t n_blocks,
                              int32_t staged_math, int32_t up, size_t workspace_bytes, sige_conv_plan_info* info)
{
    clear_error();
    const char* who = "sige_conv_plan";
    int th, tw;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    SIGE_REQUIRE(info != nullptr, SIGE_ERR_INVALID_ARG, "%s: info is required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cin > 0 && Cout > 0 && n_blocks > 0, SIGE_ERR_INVALID_ARG, "%s: Cin, Cout and n_blocks must be positive", who);
    const int ks = dt == SIGE_F32 ? 8 : 16;
    SIGE_REQUIRE(Cin % ks == 0, SIGE_ERR_UNSUPPORTED, "%s: Cin must be a multiple of %d for this dtype", who, ks);
    ConvArgs a = {};
    a.up = up;
    a.act = staged_math ? SIGE_ACT_SILU : SIGE_ACT_NONE;
    ConvPlan p;
    int pointwise = 0;
    // any 16-byte aligned non-null address stands for the workspace: nothing is dereferenced here
    void* ws = workspace_bytes ? reinterpret_cast<void*>(uintptr_t(16)) : nullptr;
    if (int rc = prepare_conv(who, dt, g, th, tw, Cin, Cout, n_blocks, n_blocks, n_blocks, a, ws, workspace_bytes, &p, &pointwise))
        return rc;
    *info = sige_conv_plan_info{};
    if (pointwise) {
        const long rows = (long)n_blocks * g->block_h * g->block_w;
        const int BM = pointwise == 3 ? 32 : 64, BN = pointwise == 2 ? 64 : 32;
        const long mt = (rows + BM - 1) / BM, nt = (Cout + BN - 1) / BN;
        const bool four = pointwise == 2 && (knob(SIGE_KNOB_CONV_POINTWISE_W4) >= 0 ? knob(SIGE_KNOB_CONV_POINTWISE_W4) != 0
                                                                                    : mt * nt > 256);
        const int W = four ? 4 : 8;
        info->kernel = 1;
        info->shape = pointwise;
        info->patch_m = BM; info->patch_n = BN;
        info->threads = 64 * W;
        info->ksplit = 1;
        info->workgroups = (int32_t)(mt * nt);
        info->lds_bytes = (int32_t)(std::max((size_t)W * BM * (BN + 4) * sizeof(float), (size_t)W * 2 * BM * 80) + 2 * BM * sizeof(int));
        return SIGE_OK;
    }
    info->kernel = 0;
    info->shape = p.cfg;
    info->patch_m = kCfg[p.cfg].M; info->patch_n = kCfg[p.cfg].N;
    info->k_steps_per_chunk = p.kc;
    info->threads = kCfg[p.cfg].WK == 8 ? 512 : 256;
    info->ksplit = p.ksplit;
    info->workgroups = (int32_t)((long)p.slabs * p.bands * p.ksplit * p.groups);
    info->lds_bytes = (int32_t)(p.lds + 2 * MAX_G * sizeof(int));
    return SIGE_OK;
}

extern "C" int sige_conv(const void* tiles, sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                         const void* packed_weight, const float* bias, const int32_t* count,
                         int32_t max_blocks, int32_t n_blocks, void* out_tiles, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    clear_error();
    const char* who = "sige_conv";
    int th, tw, nl;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(tiles && packed_weight && out_tiles, SIGE_ERR_INVALID_ARG,
                 "%s: tiles, packed_weight and out_tiles are required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cin > 0 && Cout > 0, SIGE_ERR_INVALID_ARG, "%s: Cin and Cout must be positive", who);
    const int ks = dt == SIGE_F32 ? 8 : 16;
    SIGE_REQUIRE(Cin % ks == 0, SIGE_ERR_UNSUPPORTED, "%s: Cin must be a multiple of %d for this dtype", who, ks);
    SIGE_REQUIRE(aligned16(tiles) && aligned16(packed_weight), SIGE_ERR_UNSUPPORTED,
                 "%s: tiles and packed_weight must be 16-byte aligned", who);
    if (nl == 0) return SIGE_OK;
    ConvArgs a = {};
    a.tiles = tiles; a.w = packed_weight; a.bias = bias; a.out = out_tiles; a.count = count;
    return run_conv(who, dt, g, th, tw, Cin, Cout, max_blocks, n_blocks, nl, a, workspace, workspace_bytes, stream);
}

extern "C" int sige_conv_geglu(const void* tiles, sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                               const void* packed_weight, const float* bias, const int32_t* count,
                               int32_t max_blocks, int32_t n_blocks, void* out_tiles, void* stream)
{
    clear_error();
    const char* who = "sige_conv_geglu";
    int th, tw, nl;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(tiles && packed_weight && out_tiles, SIGE_ERR_INVALID_ARG,
                 "%s: tiles, packed_weight and out_tiles are required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cin > 0 && Cout > 0, SIGE_ERR_INVALID_ARG, "%s: Cin and Cout must be positive", who);
    const int ks = dt == SIGE_F32 ? 8 : 16;
    SIGE_REQUIRE(Cin % ks == 0, SIGE_ERR_UNSUPPORTED, "%s: Cin must be a multiple of %d for this dtype", who, ks);
    SIGE_REQUIRE(Cout % 8 == 0, SIGE_ERR_UNSUPPORTED, "%s: Cout must be a multiple of 8 (values and gates come in groups of 8)", who);
    SIGE_REQUIRE(aligned16(tiles) && aligned16(packed_weight), SIGE_ERR_UNSUPPORTED,
                 "%s: tiles and packed_weight must be 16-byte aligned", who);
    if (nl == 0) return SIGE_OK;
    ConvArgs a = {};
    a.tiles = tiles; a.w = packed_weight; a.bias = bias; a.out = out_tiles; a.count = count;
    a.glu = 1;
    return run_conv(who, dt, g, th, tw, Cin, 2 * Cout, max_blocks, n_blocks, nl, a, nullptr, 0, stream);
}

extern "C" int sige_conv_scatter(const void* tiles, sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                                 const void* packed_weight, const float* bias, const int32_t* indices,
                                 const int32_t* count, int32_t max_blocks, int32_t n_blocks,
                                 const void* residual_tiles, const void* residual, int32_t res_ld, void* y,
                                 int32_t y_ld, void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    const char* who = "sige_conv_scatter";
    int th, tw, nl;
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(tiles && packed_weight && indices && y, SIGE_ERR_INVALID_ARG,
                 "%s: tiles, packed_weight, indices and y are required", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cin > 0 && Cout > 0 && y_ld >= Cout, SIGE_ERR_INVALID_ARG, "%s: need Cin, Cout > 0 and y_ld >= Cout", who);
    SIGE_REQUIRE(residual == nullptr || res_ld >= Cout, SIGE_ERR_INVALID_ARG, "%s: res_ld must be >= Cout", who);
    const int ks = dt == SIGE_F32 ? 8 : 16;
    SIGE_REQUIRE(Cin % ks == 0, SIGE_ERR_UNSUPPORTED, "%s: Cin must be a multiple of %d for this dtype", who, ks);
    SIGE_REQUIRE(aligned16(tiles) && aligned16(packed_weight), SIGE_ERR_UNSUPPORTED,
                 "%s: tiles and packed_weight must be 16-byte aligned", who);
    if (nl == 0) return SIGE_OK;
    ConvArgs a = {};
    a.tiles = tiles; a.w = packed_weight; a.bias = bias; a.count = count; a.indices = indices;
    a.res_tiles = residual_tiles; a.res_full = residual; a.y = y;
    a.Hin = g->H_in; a.Win = g->W_in; a.pad = g->pad;
    a.Hout = g->H_out; a.Wout = g->W_out; a.y_ld = y_ld; a.res_ld = res_ld;
    return run_conv(who, dt, g, th, tw, Cin, Cout, max_blocks, n_blocks, nl, a, workspace, workspace_bytes, stream);
}

// Checks the arguments of a fused call and fills the kernel arguments (nl = 0: nothing to launch).
static int fused_conv_fill(const char* who, const void* x, sige_dtype dt, int32_t Cin, int32_t x_ld, int32_t up,
                           const sige_geom* g, const int32_t* indices, const int32_t* count, int32_t max_blocks,
                           int32_t n_blocks, const float* scale, const float* shift, sige_act act, int32_t Cout,
                           const void* packed_weight, const float* bias, const void* residual_tiles,
                           const void* residual, int32_t res_ld, void* y, int32_t y_ld, void* out_tiles,
                           const sige_act_out* act_outs, int32_t n_act_outs, ConvArgs& a, int& th, int& tw, int& nl)
{
    if (int rc = check_geom(g, who, &th, &tw)) return rc;
    if (int rc = check_blocks(count, max_blocks, n_blocks, who, &nl)) return rc;
    SIGE_REQUIRE(x && indices && packed_weight, SIGE_ERR_INVALID_ARG, "%s: x, indices and packed_weight are required", who);
    SIGE_REQUIRE((y != nullptr) != (out_tiles != nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: give either y (scatter) or out_tiles (keep the tiles), not both and not neither", who);
    SIGE_REQUIRE(dtype_ok(dt), SIGE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dt);
    SIGE_REQUIRE(Cin > 0 && Cout > 0 && x_ld >= Cin, SIGE_ERR_INVALID_ARG, "%s: need Cin, Cout > 0 and x_ld >= Cin", who);
    SIGE_REQUIRE(y == nullptr || y_ld >= Cout, SIGE_ERR_INVALID_ARG, "%s: y_ld must be >= Cout", who);
    SIGE_REQUIRE(residual == nullptr || res_ld >= Cout, SIGE_ERR_INVALID_ARG, "%s: res_ld must be >= Cout", who);
    SIGE_REQUIRE(y != nullptr || (residual_tiles == nullptr && residual == nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: residuals are added by the scatter; they need y", who);
    SIGE_REQUIRE((scale == nullptr) == (shift == nullptr), SIGE_ERR_INVALID_ARG,
                 "%s: scale and shift must be given together", who);
    SIGE_REQUIRE(act_ok((int)act), SIGE_ERR_INVALID_ARG, "%s: unknown activation %d", who, (int)act);
    SIGE_REQUIRE(up == 0 || up == 1, SIGE_ERR_INVALID_ARG, "%s: up must be 0 or 1", who);
    SIGE_REQUIRE(up == 0 || (g->H_in % 2 == 0 && g->W_in % 2 == 0), SIGE_ERR_INVALID_ARG,
                 "%s: up-sampled input size must be even", who);
    const int ks = dt == SIGE_F32 ? 8 : 16;
    const size_t s = dtype_size(dt);
    SIGE_REQUIRE(Cin % ks == 0, SIGE_ERR_UNSUPPORTED, "%s: Cin must be a multiple of %d for this dtype", who, ks);
    SIGE_REQUIRE((x_ld * s) % 16 == 0 && aligned16(x) && aligned16(packed_weight), SIGE_ERR_UNSUPPORTED,
                 "%s: x and packed_weight must be 16-byte aligned and x_ld a multiple of %zu elements", who, 16 / s);
    SIGE_REQUIRE(n_act_outs >= 0 && n_act_outs <= SIGE_MAX_ACT_OUTS && (n_act_outs == 0 || act_outs != nullptr),
                 SIGE_ERR_INVALID_ARG, "%s: between 0 and %d activated copies", who, SIGE_MAX_ACT_OUTS);
    SIGE_REQUIRE(n_act_outs == 0 || y != nullptr, SIGE_ERR_INVALID_ARG,
                 "%s: activated copies are written beside the scatter; they need y", who);
    if (n_act_outs > 0) {
        // they are written from the 16-byte path of the epilogue only
        SIGE_REQUIRE((Cout * s) % 16 == 0 && (y_ld * s) % 16 == 0 && aligned16(y) &&
                     (residual == nullptr || ((res_ld * s) % 16 == 0 && aligned16(residual))) &&
                     (residual_tiles == nullptr || aligned16(residual_tiles)),
                     SIGE_ERR_UNSUPPORTED, "%s: activated copies need 16-byte channel runs in y and the residuals", who);
        for (int j = 0; j < n_act_outs; ++j) {
            const sige_act_out& o = act_outs[j];
            SIGE_REQUIRE(o.y != nullptr && o.y_ld >= Cout && (o.scale == nullptr) == (o.shift == nullptr) &&
                         act_ok((int)o.act), SIGE_ERR_INVALID_ARG, "%s: bad activated copy %d", who, j);
            SIGE_REQUIRE((o.y_ld * s) % 16 == 0 && aligned16(o.y), SIGE_ERR_UNSUPPORTED,
                         "%s: activated copy %d must be 16-byte aligned with a pixel stride that is a multiple of %zu elements",
                         who, j, 16 / s);
        }
    }
    a = ConvArgs{};
    a.n_ao = n_act_outs;
    for (int j = 0; j < n_act_outs; ++j) {
        a.ao[j].y = act_outs[j].y; a.ao[j].scale = act_outs[j].scale; a.ao[j].shift = act_outs[j].shift;
        a.ao[j].ld = act_outs[j].y_ld; a.ao[j].act = (int)act_outs[j].act;
    }
    a.w = packed_weight; a.bias = bias; a.out = out_tiles; a.count = count;
    a.x = x; a.indices = indices; a.scale = scale; a.shift = shift;
    a.res_tiles = residual_tiles; a.res_full = residual; a.y = y;
    a.Hin = g->H_in; a.Win = g->W_in; a.x_ld = x_ld; a.up = up; a.pad = g->pad; a.act = (int)act;
    a.Hout = g->H_out; a.Wout = g->W_out; a.y_ld = y_ld; a.res_ld = res_ld;
    return SIGE_OK;
}

extern "C" int sige_fused_conv(const void* x, sige_dtype dt, int32_t Cin, int32_t x_ld, int32_t up,
                               const sige_geom* g, const int32_t* indices, const int32_t* count,
                               int32_t max_blocks, int32_t n_blocks, const float* scale, const float* shift,
                               sige_act act, int32_t Cout, const void* packed_weight, const float* bias,
                               const void* residual_tiles, const void* residual, int32_t res_ld, void* y,
                               int32_t y_ld, void* out_tiles, const sige_act_out* act_outs, int32_t n_act_outs,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    clear_error();
    const char* who = "sige_fused_conv";
    ConvArgs a;
    int th, tw, nl;
    if (int rc = fused_conv_fill(who, x, dt, Cin, x_ld, up, g, indices, count, max_blocks, n_blocks, scale, shift, act,
                                 Cout, packed_weight, bias, residual_tiles, residual, res_ld, y, y_ld, out_tiles,
                                 act_outs, n_act_outs, a, th, tw, nl))
        return rc;
    if (nl == 0) return SIGE_OK;
    return run_conv(who, dt, g, th, tw, Cin, Cout, max_blocks, n_blocks, nl, a, workspace, workspace_bytes, stream);
}

// Both pair entry points.  marks == nullptr: the calls bring their lists.  Otherwise marks[i] is the list
// of call i as the marking pass left it (flags set, list not built).
static int fused_pair(const char* who, const sige_fused_conv_call* first, const sige_fused_conv_call* second,
                      const sige_block_list* marks, void* stream)
{
    SIGE_REQUIRE(first && second, SIGE_ERR_INVALID_ARG, "%s: two calls are required", who);
    const sige_fused_conv_call* c[2] = {first, second};
    ConvArgs a[2];
    ConvPlan p[2];
    int th[2], tw[2], nl[2], pw[2] = {0, 0};
    long nb[2] = {0, 0};
    if (marks != nullptr) {
        for (int i = 0; i < 2; ++i) {
            const sige_block_list& L = marks[i];
            SIGE_REQUIRE(c[i]->g != nullptr && memcmp(c[i]->g, &L.g, sizeof(sige_geom)) == 0, SIGE_ERR_INVALID_ARG,
                         "%s: call %d and its marked list differ in geometry", who, i);
            SIGE_REQUIRE(L.indices != nullptr && L.count != nullptr && c[i]->indices == L.indices &&
                             c[i]->count == L.count && c[i]->max_blocks == L.max_blocks,
                         SIGE_ERR_INVALID_ARG, "%s: call %d must read the list that its marked list describes", who, i);
            SIGE_REQUIRE(c[i]->n_blocks < 0, SIGE_ERR_INVALID_ARG,
                         "%s: the block count of call %d is not known to the host yet (n_blocks must be -1)", who, i);
            SIGE_REQUIRE(L.workspace != nullptr && L.workspace_bytes >= sige_reduce_mask_workspace_bytes(&L.g) &&
                             (reinterpret_cast<uintptr_t>(L.workspace) & 15u) == 0,
                         SIGE_ERR_INVALID_ARG, "%s: list %d needs its 16-byte aligned flag workspace", who, i);
        }
        SIGE_REQUIRE(marks[0].workspace != marks[1].workspace, SIGE_ERR_INVALID_ARG, "%s: the lists share a workspace", who);
    }
    for (int i = 0; i < 2; ++i) {
        if (int rc = fused_conv_fill(who, c[i]->x, c[i]->dt, c[i]->Cin, c[i]->x_ld, c[i]->up, c[i]->g, c[i]->indices,
                                     c[i]->count, c[i]->max_blocks, c[i]->n_blocks, c[i]->scale, c[i]->shift,
                                     c[i]->act, c[i]->Cout, c[i]->packed_weight, c[i]->bias, c[i]->residual_tiles,
                                     c[i]->residual, c[i]->res_ld, c[i]->y, c[i]->y_ld, c[i]->out_tiles,
                                     c[i]->act_outs, c[i]->n_act_outs, a[i], th[i], tw[i], nl[i]))
            return rc;
        if (nl[i] == 0) continue;
        if (int rc = prepare_conv(who, c[i]->dt, c[i]->g, th[i], tw[i], c[i]->Cin, c[i]->Cout, c[i]->max_blocks,
                                  c[i]->n_blocks, nl[i], a[i], c[i]->workspace, c[i]->workspace_bytes, &p[i], &pw[i]))
            return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    // one launch when both take the 64 x 32 shape whose four waves split K, unsplit over workgroups,
    // with the same chunk: a 3x3 call first, a 1x1 call second (measured a gain up to the 1440
    // workgroups at which calls still take that shape: 23.3 vs 25.2 us; 11.4 vs 16.3 us at 560)
    const long wgs_both = nl[0] > 0 && nl[1] > 0 && !pw[0] && !pw[1]
                              ? (long)p[0].groups * p[0].bands * p[0].slabs + (long)p[1].groups * p[1].bands * p[1].slabs
                              : 0;
    const int pair_knob = knob(SIGE_KNOB_CONV_PAIR_WGS);     // most workgroups for which the calls share a launch
    const long pair_max = pair_knob >= 0 ? pair_knob : (1L << 30);
    const bool together = nl[0] > 0 && nl[1] > 0 && wgs_both <= pair_max && !pw[0] && !pw[1] && c[0]->dt == c[1]->dt && a[0].k == 3 &&
                          a[1].k == 1 && p[0].cfg == 3 && p[1].cfg == 3 && p[0].ksplit == 1 && p[1].ksplit == 1 &&
                          p[0].kc == p[1].kc && (p[0].kc == 8 || p[0].kc == 4);
    bool scan = false;
    if (marks != nullptr) {
        // the one-launch kernel builds the lists itself when a workgroup can scan a whole block grid
        // (1024 flags); otherwise the compaction pass runs first and the calls read its lists
        scan = together;
        for (int i = 0; i < 2; ++i) {
            const sige_geom& g = marks[i].g;
            const long nbx = (g.W_out + g.block_w - 1) / g.block_w, nby = (g.H_out + g.block_h - 1) / g.block_h;
            nb[i] = nbx * nby;
            scan = scan && nb[i] <= 1024;
            a[i].mk_flags = (uint8_t*)marks[i].workspace;
            a[i].mk_half = (int)((nb[i] + 15) & ~15L);
            a[i].mk_indices = marks[i].indices;
            a[i].mk_count = marks[i].count;
            a[i].mk_nb = (int)nb[i];
            a[i].mk_nbx = (int)nbx;
            a[i].d_mk_nbx = fast_div((int)nbx);
        }
        if (!scan)
            if (int rc = compact_marked_lists(who, marks, 2, st)) return rc;
    }
    if (together) {
        const sige_dtype dt = c[0]->dt;
        return dt == SIGE_F32 ? launch_pair<float>(a[0], p[0], a[1], p[1], scan, st)
               : dt == SIGE_F16 ? launch_pair<f16>(a[0], p[0], a[1], p[1], scan, st)
                                : launch_pair<bf16>(a[0], p[0], a[1], p[1], scan, st);
    }
    for (int i = 0; i < 2; ++i) {
        if (nl[i] == 0) continue;
        if (int rc = launch_prepared(c[i]->dt, a[i], p[i], pw[i], nl[i], st)) return rc;
    }
    return SIGE_OK;
}

extern "C" int sige_fused_conv_pair(const sige_fused_conv_call* first, const sige_fused_conv_call* second,
                                    void* stream)
{
    clear_error();
    return fused_pair("sige_fused_conv_pair", first, second, nullptr, stream);
}

extern "C" int sige_fused_conv_pair_marked(const sige_fused_conv_call* first, const sige_fused_conv_call* second,
                                           const sige_block_list* marked, void* stream)
{
    clear_error();
    const char* who = "sige_fused_conv_pair_marked";
    SIGE_REQUIRE(marked != nullptr, SIGE_ERR_INVALID_ARG, "%s: the two marked lists are required", who);
    return fused_pair(who, first, second, marked, stream);
}
