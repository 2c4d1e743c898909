/*
 * sige.h - C ABI of the MI355X (gfx950) library for spatially sparse inference:
 * the cached-activation block-sparse convolution and the sparse-query attention
 * of "Efficient Spatially Sparse Inference for Conditional GANs and Diffusion
 * Models" (Sec. 3.1-3.2, Fig. "method", Fig. "pipeline" (b), Fig. "sige-attention").
 *
 * Conventions shared by every entry point
 *  - Tensors are batch 1, NHWC: an activation is [H][W][C] with C fastest.  Where
 *    a pixel stride `ld` (in elements, >= C) is given, the tensor may be a channel
 *    slice of a wider buffer; C*size and ld*size must be multiples of 16 bytes
 *    and base pointers 16-byte aligned unless a function says otherwise.
 *  - ALL pointers are DEVICE pointers owned by the caller, except `sige_geom*`
 *    (host) and where marked host.  The library allocates nothing, keeps no
 *    state between calls (but for the overrides of sige_set_knob, which tests and tuning
 *    runs use) and only enqueues work on the HIP stream passed as
 *    `void* stream` (a hipStream_t; NULL = the default stream).  No call
 *    synchronises.
 *  - Return value: SIGE_OK or an error code; argument errors are detected on the
 *    host before anything is enqueued.  sige_last_error() gives a thread-local
 *    message for the last failing call.
 *  - Block lists: int32 [max_blocks][2] = (y0, x0), the top-left OUTPUT pixel of an
 *    active block, zero-based (App. A, Fig. "scatter-gather"), row-major ascending.
 *    `count` is a device int32 holding the true number of active blocks; kernels
 *    use min(*count, max_blocks).  A host `n_blocks >= 0` sizes the launch exactly
 *    and replaces *count (count may then be NULL); n_blocks = -1 launches for
 *    max_blocks and lets surplus workgroups exit on *count.
 */
#ifndef SIGE_H
#define SIGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SIGE_OK = 0,
    SIGE_ERR_INVALID_ARG = 1, /* NULL where required, non-positive size, inconsistent geometry */
    SIGE_ERR_UNSUPPORTED = 2, /* a shape the kernels do not cover (never a silent fallback)     */
    SIGE_ERR_CAPACITY = 3,    /* host n_blocks > max_blocks, or a size beyond a stated maximum  */
    SIGE_ERR_HIP = 4          /* a HIP launch failed; message holds hipGetErrorString           */
} sige_status;

typedef enum { SIGE_F32 = 0, SIGE_F16 = 1, SIGE_BF16 = 2 } sige_dtype;
typedef enum { SIGE_ACT_NONE = 0, SIGE_ACT_SILU = 1, SIGE_ACT_RELU = 2,
               SIGE_ACT_LEAKY_RELU = 3 /* slope 0.2 for negative inputs */ } sige_act;

/* An activated copy of a layer's output (host struct, see sige_fused_conv): y is a device
 * tensor with the pixel grid of the layer's output and pixel stride y_ld >= Cout; scale and
 * shift are fp32 [Cout] device arrays (both NULL: 1 and 0).                              */
typedef struct sige_act_out {
    void* y;
    int32_t y_ld;
    const float* scale;
    const float* shift;
    sige_act act;
} sige_act_out;
#define SIGE_MAX_ACT_OUTS 3

/* Geometry of one wrapped convolution (host struct).  The output is cut into
 * block_h x block_w blocks anchored at (0,0); edge blocks may be partial.  The
 * input tile of a block is tile = (block-1)*stride + k pixels per side and starts
 * at (y0*stride - pad, x0*stride - pad): for 3x3 / stride 1 neighbouring tiles
 * overlap by 2 (Fig. "method").  Required: H_out == (H_in + 2*pad - k)/stride + 1. */
typedef struct {
    int32_t H_in, W_in;       /* spatial size the convolution reads               */
    int32_t H_out, W_out;     /* spatial size it writes                           */
    int32_t block_h, block_w; /* output block                                     */
    int32_t k, stride, pad;   /* square kernel (odd), stride >= 1, zero padding   */
} sige_geom;

/* Sec. 3.1 "Structured sparsity" + Sec. 3.2 "Tiling-based sparse convolution":
 * difference mask -> downsample -> dilate -> ordered list of active blocks.
 *
 * Mask source, exactly one of:
 *   (a_orig, a_edit): two [Hm][Wm][C] tensors of dtype dt (contiguous, ld == C);
 *       pixel marked iff for any channel !(|a_edit - a_orig| <= tau), evaluated in
 *       fp32 (NaN counts as changed).  The mask is written to mask_out, which is
 *       then REQUIRED (u8 [Hm][Wm]) and doubles as the hand-over between kernels.
 *       Fast path needs C*size % 16 == 0; other C run a scalar kernel.
 *   mask_in: a ready u8 [Hm][Wm] mask (non-zero = marked); mask_out is ignored.
 * The mask is max-pooled by 2^pool_log2 per side (a chain of 2x2 / stride-2
 * ceil-mode pools) and must then have size g->H_in x g->W_in; it is dilated by
 * `dilate` pixels (square window, clipped).  A block is active iff its input tile,
 * clipped to the image, contains a marked pixel of that mask.
 * With activations as the source, indices and count may both be NULL: only mask_out is
 * produced.
 * Outputs: indices [max_blocks][2] (rows beyond the count are left untouched; never
 * more than max_blocks rows are written) and *count = the true number of active
 * blocks, even when it exceeds max_blocks.  The block grid may hold at most
 * 131072 blocks (SIGE_ERR_CAPACITY beyond).
 * workspace: optional device scratch of sige_reduce_mask_workspace_bytes(g) bytes,
 * 16-byte aligned, which the caller zeroes ONCE before the first use and whose contents belong
 * to the library from then on (per-block flags, which every call leaves cleared for the next,
 * and two bookkeeping words); with it the marked pixels set per-block flags in parallel.  Calls that
 * share a workspace must not overlap.  NULL (or too small): one workgroup tests every
 * block - same results, slower on large grids.                                     */
int sige_reduce_mask(const void* a_orig, const void* a_edit, sige_dtype dt,
                     int32_t Hm, int32_t Wm, int32_t C, float tau,
                     const uint8_t* mask_in, int32_t pool_log2, int32_t dilate,
                     const sige_geom* g, uint8_t* mask_out,
                     int32_t* indices, int32_t max_blocks, int32_t* count,
                     void* workspace, size_t workspace_bytes, void* stream);
size_t sige_reduce_mask_workspace_bytes(const sige_geom* g);

/* sige_reduce_mask for callers that cannot allocate device memory: code that runs under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * and the same kernels as sige_reduce_mask called with a workspace (one list); the per-block flags
 * live in a scratch array built into the library (SIGE_NOALLOC_MAX_BLOCKS bytes of device memory
 * per GPU the library runs on, held until the process ends) instead of a caller workspace, and the
 * call neither allocates nor frees anything.  A block grid of more than SIGE_NOALLOC_MAX_BLOCKS
 * blocks is refused with SIGE_ERR_CAPACITY; indices and count are required (use sige_reduce_mask
 * for the mask alone).  The first call on a device resolves the array's address and clears it
 * with a small kernel on `stream`: make that call outside a stream capture.  Every call leaves
 * the flags it used zero again.  All calls on one GPU share the array: calls that overlap on one
 * GPU (different streams, different host threads) race and must be ordered by the caller.     */
#define SIGE_NOALLOC_MAX_BLOCKS 65536
int sige_reduce_mask_noalloc(const void* a_orig, const void* a_edit, sige_dtype dt,
                             int32_t Hm, int32_t Wm, int32_t C, float tau,
                             const uint8_t* mask_in, int32_t pool_log2, int32_t dilate,
                             const sige_geom* g, uint8_t* mask_out,
                             int32_t* indices, int32_t max_blocks, int32_t* count, void* stream);

/* One list of sige_reduce_mask_lists: a layer geometry, where its list goes, and its own
 * flag workspace (required here; 16-byte aligned, zeroed once by the caller, left zero by every call). */
typedef struct {
    sige_geom g;
    int32_t*  indices;          /* device [max_blocks][2]                          */
    int32_t   max_blocks;
    int32_t*  count;            /* device, one int32                               */
    void*     workspace;        /* device, sige_reduce_mask_workspace_bytes(&g)    */
    size_t    workspace_bytes;
} sige_block_list;

/* Sec. 3.2 "Tiling-based sparse convolution" for several layers at once: the layers of one
 * resolution (a 3x3 convolution and its 1x1 shortcut, a stride-2 convolution) share the
 * difference mask but have their own tiles, hence their own lists.  Same mask sources,
 * pooling, dilation and results as n_lists calls of sige_reduce_mask with the same
 * arguments; the activations are streamed once and every marked pixel sets the flags of
 * all lists.  lists is a HOST array of 1..4 entries whose geometries all have the pooled
 * mask's size as H_in x W_in; the workspaces must be distinct.                        */
int sige_reduce_mask_lists(const void* a_orig, const void* a_edit, sige_dtype dt,
                           int32_t Hm, int32_t Wm, int32_t C, float tau,
                           const uint8_t* mask_in, int32_t pool_log2, int32_t dilate,
                           const sige_block_list* lists, int32_t n_lists,
                           uint8_t* mask_out, void* stream);

/* The first half of sige_reduce_mask_lists (Sec. 3.1 difference mask; Sec. 3.2 pooling, dilation and
 * the block test): the mask is written and every list's per-block flags are set in its workspace,
 * but the ordered lists are NOT built (indices and count are not touched).  The second half -
 * flags to row-major list, flags cleared - is done by the consumer: sige_fused_conv_pair_marked.
 * On this part a dependent kernel launch costs more than the compaction's work, so a step that
 * consists of one reduction and one layer saves a launch this way.  Every call must be followed by
 * exactly one consumer of the same lists before the workspaces are used again (a second marking
 * pass in between would add its flags to the first's).  Arguments and errors as for
 * sige_reduce_mask_lists; every list needs its workspace.                                   */
int sige_mark_blocks(const void* a_orig, const void* a_edit, sige_dtype dt,
                     int32_t Hm, int32_t Wm, int32_t C, float tau,
                     const uint8_t* mask_in, int32_t pool_log2, int32_t dilate,
                     const sige_block_list* lists, int32_t n_lists,
                     uint8_t* mask_out, void* stream);

/* Fig. "method" Gather, with Sec. 3.2 "Pre-computing normalization parameters" and
 * "Kernel fusion" folded in:
 *   tiles[n][i][j][c] = act(scale[c] * x[y][x][c] + shift[c]),
 *   (y, x) = (y0*stride - pad + i, x0*stride - pad + j), and literally 0 where (y, x)
 *   lies outside g->H_in x g->W_in (padding applies to the activated tensor).
 * x is [H_in >> up][W_in >> up] pixels of x_ld elements; up = 1 reads a nearest-
 * neighbour x2 up-sampled view (source pixel = (y >> 1, x >> 1)), up = 0 reads x
 * itself.  scale/shift: fp32 [C], both NULL = identity.  Arithmetic in fp32, one
 * rounding to dt.  tiles: [max_blocks][tile_h][tile_w][C] contiguous; only the
 * first min(count, max_blocks) tiles are written.  Here and in every call below that
 * takes a block list: indices holds max_blocks rows, all readable (the kernels fetch
 * row n together with the count; rows beyond the count may hold anything).          */
int sige_gather(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, int32_t up,
                const sige_geom* g, const int32_t* indices, const int32_t* count,
                int32_t max_blocks, int32_t n_blocks,
                const float* scale, const float* shift, sige_act act,
                void* tiles, void* stream);

/* The gather of a spatially-adaptive normalisation layer (the conditional-GAN generator of
 * Sec. 4.1 "Models"; Sec. 3.2 "Pre-computing normalization parameters": the instance-norm
 * statistics of the original activation are cached and folded into scale / shift, fp32 [C]):
 *   tiles[n][i][j][c] = act((scale[c] * x[y][x][c] + shift[c]) * (1 + gamma[y][x][c]) + beta[y][x][c]),
 * zero outside the image.  mod is the per-pixel modulation tensor [H_in][W_in] with pixel
 * stride mod_ld elements, gamma in channels 0..C-1 and beta in channels C..2C-1 (the output of
 * the modulation convolutions, itself updated sparsely); it lives at the resolution the
 * convolution reads, also when up = 1 (x is then the half-resolution tensor).  Everything
 * else as in sige_gather; scale / shift NULL = identity.                              */
int sige_gather_modulated(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, int32_t up,
                          const sige_geom* g, const int32_t* indices, const int32_t* count,
                          int32_t max_blocks, int32_t n_blocks,
                          const float* scale, const float* shift,
                          const void* mod, int32_t mod_ld, sige_act act,
                          void* tiles, void* stream);

/* Fig. "method": the convolution F_l applied to the stacked tiles (valid, i.e. no
 * padding inside a tile), with bias (Fig. "pipeline" (b)):
 *   out[n][py][px][o] = bias[o] + sum_{ky,kx,c} W[o][c][ky][kx] *
 *                       tiles[n][py*stride+ky][px*stride+kx][c].
 * An implicit GEMM on the matrix cores with fp32 accumulation, one rounding to dt.
 * packed_weight comes from sige_pack_weight for the same (dt, Cout, Cin, k); bias
 * fp32 [Cout] or NULL.  Cin must be a multiple of 16 (f16/bf16) or 8 (f32).
 * out_tiles: [max_blocks][block_h][block_w][Cout] contiguous.
 * workspace: optional device scratch (16-byte aligned, any contents, no state kept between
 * calls; sige_conv_workspace_bytes gives the size that allows every split).  With it a call
 * that has few active blocks but many input channels (the low-resolution layers of a UNet)
 * is cut along K over more workgroups, which leave fp32 partial sums there; a second kernel
 * adds them in a fixed order.  Results are deterministic for a given workspace size; with
 * and without a workspace they may differ in the last bit of the fp32 sum.  Calls that
 * share a workspace must not overlap.  NULL: never split.                            */
int sige_conv(const void* tiles, sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
              const void* packed_weight, const float* bias,
              const int32_t* count, int32_t max_blocks, int32_t n_blocks,
              void* out_tiles, void* workspace, size_t workspace_bytes, void* stream);
/* Bytes of workspace with which sige_conv / sige_fused_conv can split K as far as they would
 * for any number of blocks up to max_blocks (0 when they never split this layer).    */
size_t sige_conv_workspace_bytes(sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                                 int32_t max_blocks);

/* Which kernel a convolution call would run (host only, nothing is enqueued): for tests that must
 * know which code path they cover and for tuning.  n_blocks = the number of blocks the launch is
 * sized for; staged_math != 0 when Scale+Shift or an activation is applied on the way into LDS;
 * up as in sige_fused_conv; workspace_bytes as the call would get (0 = none).
 *   kernel             0 = tiled implicit GEMM, 1 = the 1x1 kernel for few rows
 *   shape              tiled: 0 = 128x128, 1 = 128x64, 2 = 64x64, 3 = 64x32 with four waves splitting K,
 *                      4 = 64x32 and 5 = 32x32 with eight waves splitting K; few rows: 1 = 64x32, 2 = 64x64,
 *                      3 = 32x32
 *   patch_m, patch_n   output rows (pixels) x channels per workgroup
 *   k_steps_per_chunk  MFMA K steps per staged channel chunk (tiled kernel)
 *   ksplit             workgroups sharing one output patch along K (> 1: a second kernel adds them)
 *   workgroups, threads, lds_bytes (dynamic + static) of the launch                              */
typedef struct {
    int32_t kernel, shape, patch_m, patch_n, k_steps_per_chunk, ksplit, workgroups, threads, lds_bytes;
} sige_conv_plan_info;
int sige_conv_plan(sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout, int32_t n_blocks,
                   int32_t staged_math, int32_t up, size_t workspace_bytes, sige_conv_plan_info* info);

/* Fig. "pipeline" (b) Scatter: y holds the cached F_l(A_orig) on entry and is updated
 * in place; for every active block and every in-image pixel of it
 *   y[y0+i][x0+j][o] = out_tiles[n][i][j][o] (+ residual_tiles[n][i][j][o])
 *                                            (+ residual[y0+i][x0+j][o]);
 * all other elements of y are left untouched.  Sums are taken in fp32 and rounded
 * once.  residual_tiles ([max_blocks][block_h][block_w][Cout]) and residual (a full
 * [H_out][W_out] tensor with pixel stride res_ld) may each be NULL.  Blocks are
 * disjoint, so the stores never race.  y has pixel stride y_ld.                    */
int sige_scatter(const void* out_tiles, sige_dtype dt, const sige_geom* g, int32_t Cout,
                 const int32_t* indices, const int32_t* count, int32_t max_blocks, int32_t n_blocks,
                 const void* residual_tiles, const void* residual, int32_t res_ld,
                 void* y, int32_t y_ld, void* stream);

/* sige_conv on the stacked tiles with the gated GELU of a feed-forward layer (sige_geglu) folded into
 * its epilogue: the convolution has 2*Cout output channels, laid out in groups of 16 = 8 value
 * channels followed by their 8 gate channels (pack the OIHW weight with its rows in that order:
 * rows 16j..16j+7 = value channels 8j..8j+7, rows 16j+8..16j+15 = their gates; bias likewise,
 * fp32 [2*Cout] or NULL), and
 *   out[n][py][px][c] = value_c * gelu(gate_c),  gelu(g) = g/2 * (1 + erf(g / sqrt 2)),
 * computed from the fp32 sums: the layer has ONE stored tensor, this product, rounded once (the
 * 2*Cout-channel intermediate is never stored or rounded).
 * out_tiles: [max_blocks][block_h][block_w][Cout].  Cout must be a multiple of 8.  Never splits K
 * over workgroups (no workspace).  Other arguments as in sige_conv.                        */
int sige_conv_geglu(const void* tiles, sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                    const void* packed_weight, const float* bias,
                    const int32_t* count, int32_t max_blocks, int32_t n_blocks,
                    void* out_tiles, void* stream);

/* Sec. 3.2 "Kernel fusion", the output half: sige_conv on the stacked tiles with sige_scatter
 * folded into its epilogue - the output tiles never touch HBM.  For layers whose input tiles
 * already exist (the token-wise layers between Gather and Scatter of Fig. "sige-attention":
 * the projection that leaves an attention block, keys and values on their way into the
 * caches).  Arguments as in sige_conv and sige_scatter; the residuals are added to the fp32
 * sums and the result is rounded to dt once (Scatter with Block Residual, App. A.2: the
 * layer's stored output is the convolution plus its residuals).  workspace as in sige_conv. */
int sige_conv_scatter(const void* tiles, sige_dtype dt, const sige_geom* g, int32_t Cin, int32_t Cout,
                      const void* packed_weight, const float* bias,
                      const int32_t* indices, const int32_t* count, int32_t max_blocks, int32_t n_blocks,
                      const void* residual_tiles, const void* residual, int32_t res_ld,
                      void* y, int32_t y_ld, void* workspace, size_t workspace_bytes, void* stream);

/* Sec. 3.2 "Kernel fusion" taken to its end on this hardware: Gather (with Scale+Shift and
 * the nonlinearity), the convolution and Scatter (with the residual additions) in ONE
 * kernel.  The input tile of each active block is gathered from x straight into LDS,
 * multiplied on the matrix cores, and the result goes straight into y - the stacked tiles
 * never touch HBM.  Arguments as in sige_gather / sige_conv / sige_scatter.  Residuals are
 * added to the fp32 sums and the result is rounded to dt once (Scatter with Block Residual,
 * App. A.2: the layer's stored output is the convolution plus its residuals; the three calls
 * round the stored output tiles first and once more after the addition, so with residuals
 * the fused result may differ from theirs in the last place).  Without residuals the results
 * are bit-identical to calling those three in sequence whenever both run the same kernel
 * shape (always, except for a 1x1 convolution with Scale+Shift or an activation, where
 * sige_conv alone may take the few-row kernel and the fp32 sums are added in another order).
 * Exactly one of
 *   y         - scatter into the cached output, in place (residuals allowed), or
 *   out_tiles - keep the output tiles [max_blocks][block_h][block_w][Cout] (a shortcut
 *               branch whose tiles a later call adds as residual_tiles)
 * must be given.  x and y must not overlap (a tile's halo belongs to other blocks).
 * workspace: as for sige_conv (the reduction kernel then also adds the residuals and
 * scatters); bit-identity with the three calls (no residuals) holds when sige_conv gets a
 * workspace of the same size.
 * act_outs (n_act_outs of them, 0..SIGE_MAX_ACT_OUTS; scatter mode only): Sec. 3.2
 * "Pre-computing normalization parameters" makes the Scale+Shift of the NEXT layer a
 * constant per channel, so the layer that produces a tensor can apply it, and the
 * nonlinearity, to each value once instead of every gathering workgroup doing so again:
 * besides y[p][o] = v, copy j receives
 *   act_outs[j].y[p][o] = act_j(scale_j[o] * v + shift_j[o])
 * computed in fp32 from the stored (rounded) v, i.e. bit for bit what a fused gather of y
 * with the same scale, shift and activation would read.  A consumer then gathers the copy
 * without Scale+Shift.  Needs Cout * size and all pixel strides to be multiples of 16 bytes
 * (else SIGE_ERR_UNSUPPORTED).                                                        */
int sige_fused_conv(const void* x, sige_dtype dt, int32_t Cin, int32_t x_ld, int32_t up,
                    const sige_geom* g, const int32_t* indices, const int32_t* count,
                    int32_t max_blocks, int32_t n_blocks,
                    const float* scale, const float* shift, sige_act act,
                    int32_t Cout, const void* packed_weight, const float* bias,
                    const void* residual_tiles, const void* residual, int32_t res_ld,
                    void* y, int32_t y_ld, void* out_tiles,
                    const sige_act_out* act_outs, int32_t n_act_outs,
                    void* workspace, size_t workspace_bytes, void* stream);

/* Two independent fused calls handed over together, e.g. a ResBlock's 3x3 convolution and its 1x1
 * shortcut, which read the same tensor through lists of the same resolution (Fig. "method"; the
 * paper's per-layer pipeline run for two layers side by side).  Each struct holds the arguments
 * of one sige_fused_conv call, with the same meaning and the same checks.  When the first is a
 * 3x3 and the second a 1x1 convolution of the same dtype and both would take the few-block kernel
 * shape without a K split over workgroups, they run as ONE kernel launch (on this part a launch
 * of a dependent kernel costs more than the work of such a call); otherwise one after the other.
 * The outputs are bit-identical to those of the two separate calls.  The two calls must not
 * write what the other reads or writes.                                                      */
typedef struct {
    const void* x; sige_dtype dt; int32_t Cin, x_ld, up;
    const sige_geom* g; const int32_t* indices; const int32_t* count;
    int32_t max_blocks, n_blocks;
    const float* scale; const float* shift; sige_act act;
    int32_t Cout; const void* packed_weight; const float* bias;
    const void* residual_tiles; const void* residual; int32_t res_ld;
    void* y; int32_t y_ld; void* out_tiles;
    const sige_act_out* act_outs; int32_t n_act_outs;
    void* workspace; size_t workspace_bytes;
} sige_fused_conv_call;
int sige_fused_conv_pair(const sige_fused_conv_call* first, const sige_fused_conv_call* second,
                         void* stream);

/* sige_fused_conv_pair on lists that sige_mark_blocks left marked: marked is a HOST array of two
 * entries, marked[i] the list of call i (same geometry; call i's indices, count and max_blocks must be
 * marked[i]'s; n_blocks must be -1, the count is not known to the host).  Same results as the
 * compaction of sige_reduce_mask_lists followed by sige_fused_conv_pair: the ordered lists and
 * their counts are stored in marked[i].indices / count as there, the workspaces are ready for the
 * next reduction or marking pass on return, the outputs are bit-identical.  When the two calls share a launch and each block grid
 * has at most 1024 blocks, the workgroups build the lists themselves from the flags (no
 * compaction launch; the workspace's second half and its phase words let the flags of this step
 * stay in place while the half for the next step is cleared); otherwise the compaction pass
 * runs first.                                                                              */
int sige_fused_conv_pair_marked(const sige_fused_conv_call* first, const sige_fused_conv_call* second,
                                const sige_block_list* marked, void* stream);

/* Fig. "sige-attention" / Sec. 3.2 "Extension to attention layers": attention for the
 * edited query tokens only, against all T keys and values (the caches with the
 * edited tokens already overwritten):
 *   o[i][h][:] = sum_t softmax_t(scale * q[i][h][:] . k[t][h][:]) * v[t][h][:].
 * q, o: [Nq][heads][d] with row strides q_ld / o_ld elements; k, v: [T][heads][d]
 * with row stride kv_ld (a row = one token, heads*d contiguous elements inside it).
 * Any dt; d * size and the strides * size multiples of 16 bytes, d <= 256.
 * Streaming (online) softmax in fp32 on the matrix cores.  fp16 feeds the probabilities
 * to the second product rounded to fp16, bf16 as the sum of two bf16 numbers (16 bits), and
 * both normalise by the sum of exactly those values; single precision (the precision of
 * the paper's experiments, Sec. 4.1) rounds nothing in between.  Nq is a host value;
 * Nq == 0 enqueues nothing.
 * workspace: optional device scratch for splitting the keys over several workgroups
 * when Nq is small; sige_sparse_attn_workspace_bytes gives the size that allows it.
 * NULL (or too small) runs without key splitting.                                 */
int sige_sparse_attn(const void* q, int32_t q_ld, const void* k, const void* v, int32_t kv_ld,
                     sige_dtype dt, int32_t Nq, int32_t T, int32_t heads, int32_t d, float scale,
                     void* o, int32_t o_ld, void* workspace, size_t workspace_bytes, void* stream);
size_t sige_sparse_attn_workspace_bytes(int32_t Nq, int32_t T, int32_t heads, int32_t d);

/* The same attention with the queries taken straight from a full-resolution tensor by
 * block list (Fig. "sige-attention": the gather of the query tokens folded into the
 * attention call): q is [H_in*W_in][heads][d] with row stride q_ld, one row per pixel;
 * query i of the call is pixel i % (block_h*block_w) (row-major inside the block) of
 * block i / (block_h*block_w), whose top-left corner is indices[2*b], indices[2*b+1];
 * Nq = n_blocks * block_h * block_w and o is the [Nq][heads][d] stacked result, as
 * above.  g must be the geometry of a 1x1, stride-1, unpadded layer; n_blocks is a
 * host value >= 0 (0 enqueues nothing).  Pixels of a block that stick out of the map
 * read the nearest pixel inside it.  Use sige_sparse_attn_workspace_bytes with that Nq.
 * With q, k and v three channel ranges of one cached tensor, one convolution
 * (sige_conv_scatter) can refresh all three for the active tokens.                  */
int sige_sparse_attn_blocks(const void* q, int32_t q_ld, const sige_geom* g, const int32_t* indices,
                            int32_t n_blocks, const void* k, const void* v, int32_t kv_ld,
                            sige_dtype dt, int32_t T, int32_t heads, int32_t d, float scale,
                            void* o, int32_t o_ld, void* workspace, size_t workspace_bytes, void* stream);

/* Sec. 3.2 "Extension to attention layers" (Fig. "sige-attention"): between Gather and
 * Scatter an attention block sees only the tokens of the active blocks, so its token-wise
 * layers run on the stacked tiles, one row per token: x is [n_rows][C] with row stride x_ld,
 * y likewise.  Rows: n_rows >= 0 from the host, or -1 = min(*count * rows_per_count,
 * max_rows) read on the device (count = the block count, rows_per_count = tokens per
 * block).  C * size and the strides must be multiples of 16 bytes.  x == y is allowed
 * for sige_token_norm (a wave reads its whole row before it writes).
 *
 * sige_token_norm: per-token layer normalisation over the C channels,
 *   y[r][c] = (x[r][c] - mean_r) / sqrt(var_r + eps) * gamma[c] + beta[c],
 * mean and biased variance of row r in fp32 (two passes over registers), gamma / beta
 * fp32 [C] or NULL (1 / 0).  At most 8 KiB per token.
 * sige_geglu: the gated GELU of a feed-forward layer, x is [n_rows][2C],
 *   y[r][c] = x[r][c] * gelu(x[r][C + c]),  gelu(g) = g/2 * (1 + erf(g / sqrt 2)).
 * (Layer norm and the gated feed-forward are the latent-diffusion transformer block's
 * operators; the paper applies the engine to that model, Sec. 4.1, without describing
 * the block.)                                                                        */
int sige_token_norm(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, const int32_t* count,
                    int32_t rows_per_count, int32_t max_rows, int32_t n_rows,
                    const float* gamma, const float* beta, float eps,
                    void* y, int32_t y_ld, void* stream);

/* The gather of Fig. "sige-attention" with the token norm above folded in: tiles[n][i][j][:]
 * = layer norm (as sige_token_norm) of pixel (y0_n + i, x0_n + j) of x, for the active blocks
 * of a geometry whose tiles are the blocks themselves (k = 1, stride 1, no padding; other
 * geometries -> SIGE_ERR_UNSUPPORTED).  x is [H_in][W_in][x_ld >= C]; tiles is
 * [max_blocks][block_h][block_w][C]; a pixel outside x counts as a row of zeros, as in
 * sige_gather.  indices / count / max_blocks / n_blocks as in sige_gather.              */
int sige_gather_token_norm(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, const sige_geom* g,
                           const int32_t* indices, const int32_t* count, int32_t max_blocks,
                           int32_t n_blocks, const float* gamma, const float* beta, float eps,
                           void* tiles, void* stream);
int sige_geglu(const void* x, sige_dtype dt, int32_t C, int32_t x_ld, const int32_t* count,
               int32_t rows_per_count, int32_t max_rows, int32_t n_rows,
               void* y, int32_t y_ld, void* stream);

/* ---- helpers beside the path --------------------------------------------------- */

/* Re-lays an OIHW weight tensor (device, dtype dt, [Cout][Cin][k][k]) into the
 * matrix-core fragment order sige_conv reads; done once per layer.                */
size_t sige_packed_weight_bytes(sige_dtype dt, int32_t Cout, int32_t Cin, int32_t k);
int sige_pack_weight(const void* w_oihw, sige_dtype dt, int32_t Cout, int32_t Cin, int32_t k,
                     void* packed, void* stream);

/* Sec. 3.2 "Pre-computing normalization parameters": group statistics of a full
 * [H][W][C] tensor (pixel stride x_ld) from the pre-computation pass, folded into
 * the per-channel Scale+Shift the gather applies:
 *   scale[c] = gamma[c] / sqrt(var_g + eps), shift[c] = beta[c] - mean_g * scale[c],
 * mean_g and the biased var_g taken over H*W*(C/groups) elements.  mean, var:
 * fp32 [groups] outputs (also used as accumulators); gamma, beta, scale, shift:
 * fp32 [C]; gamma/beta NULL = 1/0.  C % groups == 0.                              */
int sige_gn_stats(const void* x, sige_dtype dt, int32_t H, int32_t W, int32_t C, int32_t x_ld,
                  int32_t groups, const float* gamma, const float* beta, float eps,
                  float* mean, float* var, float* scale, float* shift, void* stream);

const char* sige_last_error(void);
int sige_version(void);

/* Overrides of the launch heuristics, for tests that must reach a given kernel shape and for
 * tuning runs.  This is the only state the library keeps: process-wide, read on the host when a
 * call is planned; set them while no other thread is inside a call.  value < 0 restores the
 * automatic choice (the default of every knob).  An override that a call cannot honour (a shape
 * that does not fit the layer) is ignored or ends in SIGE_ERR_UNSUPPORTED, never in a wrong
 * result.
 *   CONV_CFG           workgroup shape of the tiled convolution: 0 = 128x128, 1 = 128x64, 2 = 64x64,
 *                      3 = 64x32 with four waves splitting K; with CONV_KC >= 16 also 4 (eight waves)
 *   CONV_KC            K steps per staged channel chunk (1, 3, 4, 8; 16, 20, 32, 40 = whole-Cin shapes)
 *   CONV_SPLIT         number of workgroups that share an output patch along K (needs a workspace)
 *   CONV_HALF          most workgroups up to which the eight-wave shape takes 32-row patches
 *   CONV_SPLIT_WGS     workgroups a K split over workgroups aims for
 *   CONV_POINTWISE     the few-row 1x1 kernel: 0 = never, 1 = 64x32, 2 = 64x64, 3 = 32x32 patches
 *   CONV_POINTWISE_W4  its four-wave variant for 64x64 patches: 0 = never, 1 = always
 *   CONV_PAIR_WGS      most workgroups up to which sige_fused_conv_pair shares one launch
 *   ATTN_WGS           workgroups the key split of sige_sparse_attn aims for
 *   DIFF_LOADS         16-byte loads per lane and tensor in flight in the difference kernel (1, 2, 4)
 *   DIFF_WGS           accepted and ignored (the difference kernel runs one step per wave)
 *   CONV_DIRECT        0: the shapes whose waves do not split K send their accumulators through LDS
 *                      instead of straight from the registers
 *   CONV_LDS_PAD       bytes between the staged pixels' channel runs in LDS (a multiple of 16)        */
typedef enum {
    SIGE_KNOB_CONV_CFG = 0, SIGE_KNOB_CONV_KC = 1, SIGE_KNOB_CONV_SPLIT = 2, SIGE_KNOB_CONV_HALF = 3,
    SIGE_KNOB_CONV_SPLIT_WGS = 4, SIGE_KNOB_CONV_POINTWISE = 5, SIGE_KNOB_CONV_POINTWISE_W4 = 6,
    SIGE_KNOB_CONV_PAIR_WGS = 7, SIGE_KNOB_ATTN_WGS = 8, SIGE_KNOB_DIFF_LOADS = 9, SIGE_KNOB_DIFF_WGS = 10,
    SIGE_KNOB_CONV_DIRECT = 11, SIGE_KNOB_CONV_LDS_PAD = 12, SIGE_KNOB_COUNT = 13
} sige_knob;
int sige_set_knob(sige_knob knob, int32_t value);
int32_t sige_get_knob(sige_knob knob);

#ifdef __cplusplus
}
#endif
#endif /* SIGE_H */
