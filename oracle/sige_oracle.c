/*
 * CPU oracle for the cached-activation block-sparse convolution and the
 * sparse-query attention of Spatially Sparse Inference.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision statement
 * of what the method computes, written from the paper, and it shares nothing
 * with the HIP library: no header, no table, no helper.  Only the tests, the
 * smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * Layout everywhere: batch 1, NHWC (a tensor is [H][W][C], C fastest).
 * Floating inputs arrive as doubles that already hold storage-dtype values
 * exactly; every sum is accumulated in double; nothing is rounded here.
 *
 * Each function names the passage of the paper it restates.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Sec. 3.1 "Structured sparsity": a binary difference mask between the
 * original and the edited tensor.  A pixel is marked when any channel differs
 * by more than tau.  The subtraction is done in IEEE single precision on
 * exactly converted inputs; NaN counts as "changed".                         */
void oracle_diff_mask(const float *a_orig, const float *a_edit, int H, int W, int C,
                      float tau, uint8_t *mask)
{
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
            uint8_t m = 0;
            for (int c = 0; c < C; ++c) {
                size_t i = ((size_t)y * W + x) * C + c;
                volatile float d = a_edit[i] - a_orig[i];
                if (!(fabsf(d) <= tau)) m = 1;
            }
            mask[(size_t)y * W + x] = m;
        }
}

/* Sec. 3.2 "Tiling-based sparse convolution": the mask is downsampled to every
 * feature-map scale.  One level = 2x2 max-pool, stride 2, ceil mode (a partial
 * window at the border still produces an output pixel).                      */
void oracle_downsample(const uint8_t *m, int H, int W, uint8_t *out)
{
    int Ho = (H + 1) / 2, Wo = (W + 1) / 2;
    for (int y = 0; y < Ho; ++y)
        for (int x = 0; x < Wo; ++x) {
            uint8_t v = 0;
            for (int dy = 0; dy < 2; ++dy)
                for (int dx = 0; dx < 2; ++dx) {
                    int yy = 2 * y + dy, xx = 2 * x + dx;
                    if (yy < H && xx < W && m[(size_t)yy * W + xx]) v = 1;
                }
            out[(size_t)y * Wo + x] = v;
        }
}

/* Sec. 3.2: the downsampled mask is dilated by r pixels.  Square window of
 * edge 2r+1, clipped at the border.                                          */
void oracle_dilate(const uint8_t *m, int H, int W, int r, uint8_t *out)
{
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
            uint8_t v = 0;
            for (int dy = -r; dy <= r; ++dy)
                for (int dx = -r; dx <= r; ++dx) {
                    int yy = y + dy, xx = x + dx;
                    if (yy >= 0 && yy < H && xx >= 0 && xx < W && m[(size_t)yy * W + xx]) v = 1;
                }
            out[(size_t)y * W + x] = v;
        }
}

/* Sec. 3.2 and Fig. "method": the output is cut into blocks of bh x bw anchored
 * at (0,0); a block is active when the input region its outputs depend on
 * (its footprint, (b-1)*stride+k wide, starting at y0*stride-pad) contains a
 * marked pixel.  The list holds the top-left output corner of every active
 * block, zero-based (App. A, Fig. "scatter-gather"), in row-major order.
 * Returns the number of active blocks; idx must hold 2*ceil(Ho/bh)*ceil(Wo/bw). */
int oracle_active_blocks(const uint8_t *m, int Hin, int Win, int Hout, int Wout,
                         int bh, int bw, int k, int stride, int pad, int32_t *idx)
{
    int n = 0;
    for (int y0 = 0; y0 < Hout; y0 += bh)
        for (int x0 = 0; x0 < Wout; x0 += bw) {
            int fy = y0 * stride - pad, fx = x0 * stride - pad;
            int th = (bh - 1) * stride + k, tw = (bw - 1) * stride + k;
            int any = 0;
            for (int y = fy; y < fy + th; ++y)
                for (int x = fx; x < fx + tw; ++x)
                    if (y >= 0 && y < Hin && x >= 0 && x < Win && m[(size_t)y * Win + x]) any = 1;
            if (any) { idx[2 * n] = y0; idx[2 * n + 1] = x0; ++n; }
        }
    return n;
}

/* Sec. 3.2 "Pre-computing normalization parameters": group statistics of a
 * full tensor (mean and biased variance over H*W*(C/G) elements per group).  */
void oracle_gn_stats(const double *x, int H, int W, int C, int G, double *mean, double *var)
{
    int cg = C / G;
    for (int g = 0; g < G; ++g) {
        double s = 0.0;
        for (size_t p = 0; p < (size_t)H * W; ++p)
            for (int c = g * cg; c < (g + 1) * cg; ++c) s += x[p * C + c];
        double mu = s / ((double)H * W * cg), q = 0.0;
        for (size_t p = 0; p < (size_t)H * W; ++p)
            for (int c = g * cg; c < (g + 1) * cg; ++c) {
                double d = x[p * C + c] - mu;
                q += d * d;
            }
        mean[g] = mu;
        var[g] = q / ((double)H * W * cg);
    }
}

/* Sec. 3.2 "Pre-computing normalization parameters" + "Kernel fusion": with the
 * statistics of the ORIGINAL activation the normalisation is a per-channel
 * Scale+Shift, followed by the nonlinearity (0 none, 1 SiLU, 2 ReLU).
 * scale/shift may be NULL (identity).                                        */
void oracle_scale_shift_act(const double *x, int H, int W, int C, const double *scale,
                            const double *shift, int act, double *z)
{
    for (size_t p = 0; p < (size_t)H * W; ++p)
        for (int c = 0; c < C; ++c) {
            double v = x[p * C + c];
            if (scale) v = scale[c] * v + shift[c];
            if (act == 1) v = v / (1.0 + exp(-v));
            else if (act == 2) v = v > 0.0 ? v : 0.0;
            else if (act == 3) v = v > 0.0 ? v : 0.2 * v;   /* leaky ReLU, slope 0.2 */
            z[p * C + c] = v;
        }
}

/* Sec. 3.1 "Preliminary": F(A) = W * A + b, the plain definition of a 2-D
 * convolution (cross-correlation, as every deep-learning framework defines
 * it) with zero padding.  w is OIHW.  bias may be NULL.
 * If pixels != NULL only the npix output pixels (y,x pairs) are computed and
 * y is [npix][Cout]; otherwise y is the full [Hout][Wout][Cout].             */
static void conv_pixel(const double *z, int Hin, int Win, int Cin, const double *w,
                       const double *bias, int Cout, int k, int stride, int pad,
                       int y, int x, double *out)
{
    for (int o = 0; o < Cout; ++o) {
        double acc = bias ? bias[o] : 0.0;
        for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
                int yy = y * stride + ky - pad, xx = x * stride + kx - pad;
                if (yy < 0 || yy >= Hin || xx < 0 || xx >= Win) continue; /* zero padding */
                const double *zp = z + ((size_t)yy * Win + xx) * Cin;
                for (int c = 0; c < Cin; ++c)
                    acc += w[(((size_t)o * Cin + c) * k + ky) * k + kx] * zp[c];
            }
        out[o] = acc;
    }
}

void oracle_conv2d(const double *z, int Hin, int Win, int Cin, const double *w,
                   const double *bias, int Cout, int k, int stride, int pad,
                   int Hout, int Wout, const int32_t *pixels, int npix, double *y)
{
    if (pixels) {
#pragma omp parallel for schedule(dynamic, 16)
        for (int i = 0; i < npix; ++i)
            conv_pixel(z, Hin, Win, Cin, w, bias, Cout, k, stride, pad, pixels[2 * i],
                       pixels[2 * i + 1], y + (size_t)i * Cout);
        return;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int yy = 0; yy < Hout; ++yy)
        for (int xx = 0; xx < Wout; ++xx)
            conv_pixel(z, Hin, Win, Cin, w, bias, Cout, k, stride, pad, yy, xx,
                       y + ((size_t)yy * Wout + xx) * Cout);
}

/* Fig. "pipeline" (b): the edited output is the cached original output with the
 * active output blocks replaced by the newly computed values.  Blocks are
 * clipped at the image border.                                               */
void oracle_select_blocks(const double *y_new, const double *y_cache, int H, int W, int C,
                          const int32_t *idx, int n, int bh, int bw, double *out)
{
    memcpy(out, y_cache, (size_t)H * W * C * sizeof(double));
    for (int b = 0; b < n; ++b)
        for (int y = idx[2 * b]; y < idx[2 * b] + bh && y < H; ++y)
            for (int x = idx[2 * b + 1]; x < idx[2 * b + 1] + bw && x < W; ++x)
                memcpy(out + ((size_t)y * W + x) * C, y_new + ((size_t)y * W + x) * C,
                       (size_t)C * sizeof(double));
}

/* Sec. 3.2 "Extension to attention layers": for each query token and head,
 * softmax(q K^T * scale) V over ALL T keys.  q,o: [Nq][heads][d];
 * k,v: [T][heads][d].  Max-subtracted softmax, all in double.                */
void oracle_attention(const double *q, const double *k, const double *v, int Nq, int T,
                      int heads, int d, double scale, double *o)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < Nq; ++i) {
        double *s = (double *)malloc((size_t)T * sizeof(double));
        for (int h = 0; h < heads; ++h) {
            const double *qi = q + ((size_t)i * heads + h) * d;
            double mx = -INFINITY;
            for (int t = 0; t < T; ++t) {
                const double *kt = k + ((size_t)t * heads + h) * d;
                double a = 0.0;
                for (int e = 0; e < d; ++e) a += qi[e] * kt[e];
                s[t] = a * scale;
                if (s[t] > mx) mx = s[t];
            }
            double den = 0.0;
            for (int t = 0; t < T; ++t) { s[t] = exp(s[t] - mx); den += s[t]; }
            double *oi = o + ((size_t)i * heads + h) * d;
            for (int e = 0; e < d; ++e) {
                double a = 0.0;
                for (int t = 0; t < T; ++t) a += s[t] * v[((size_t)t * heads + h) * d + e];
                oi[e] = a / den;
            }
        }
        free(s);
    }
}
