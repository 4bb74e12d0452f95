/*
 * CPU oracle for direct sparse convolution -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct reference used by the tests, the smoke check and the
 * bench's cpu_baseline leg.  It shares no code, header, table or helper with the HIP
 * library and is never called by the product path.
 *
 * What is computed (paper's notation, Table 1: N batch, M filters, C channels, H/W ifmap,
 * R/S filter, E/F ofmap):
 *   - oracle_conv / oracle_conv_points: the convolution layer's definition, Eq. (1) /
 *     Algorithm 1 (cross-correlation, no filter flip), generalised with symmetric zero
 *     padding done by a bounds check (no padded buffer) and a stride on the output
 *     coordinate.  The method changes no result ("no effect on accuracy", Section 4), so
 *     the oracle is the definition itself on the dense filter bank scattered from CSR.
 *     Accumulation is fp64; B = sum |w*x| is returned beside it for the error bound.
 *   - oracle_stretch: weight stretching (Section 3.1): column j=(c*R+r)*S+s of the M x CRS
 *     filter matrix becomes the CHW layout offset f(c,r,s)=(c*Hin+r)*Win+s on the padded
 *     input dims.
 *   - oracle_pad: the zero-padded 1-D input array of Section 3.1 (the pad_in step of
 *     Section 4.2).
 *   - oracle_sconv_alg2: the layer in its stretched form (Section 3.1, the result of
 *     Algorithm 2): per output element, the sum over the CSR row's entries of value times
 *     the padded 1-D array at (stretched offset + f(0,h,w)), fp64 sum.  It must agree with
 *     oracle_conv; that agreement pins the readings of padding, stride and f(0,h,w).
 *
 * All tensors are contiguous NCHW / MCRS, indices int32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F_BIAS 1u
#define ORACLE_F_RELU 2u

typedef struct {
    int N, C, H, W, M, R, S, stride, pad;
} shape_t;

static int out_h(const shape_t *p) { return (p->H + 2 * p->pad - p->R) / p->stride + 1; }
static int out_w(const shape_t *p) { return (p->W + 2 * p->pad - p->S) / p->stride + 1; }

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Dense filter bank Wd[m][c][r][s] (fp64) from CSR rows over columns j=(c*R+r)*S+s.
 * Duplicate entries add up, as Algorithm 2's "+=" implies.  Returns -1 on a bad index. */
int oracle_csr_to_dense(int M, int C, int R, int S, const int32_t *rowptr, const int32_t *colidx,
                        const float *value, double *Wd)
{
    const int64_t cols = (int64_t)C * R * S;
    memset(Wd, 0, sizeof(double) * (size_t)M * (size_t)cols);
    for (int m = 0; m < M; ++m) {
        for (int32_t j = rowptr[m]; j < rowptr[m + 1]; ++j) {
            int32_t col = colidx[j];
            if (col < 0 || col >= cols) return -1;
            int c = col / (R * S);
            int r = (col % (R * S)) / S;
            int s = col % S;
            Wd[(((int64_t)m * C + c) * R + r) * S + s] += (double)value[j];
        }
    }
    return 0;
}

/* One output element by Eq. (1): sum over c, r, s of I[n][c][h*stride+r-pad][w*stride+s-pad]
 * * W[m][c][r][s], out-of-range input coordinates contributing zero. */
static void conv_point(const shape_t *p, const float *in, const double *Wd, int n, int m, int h,
                       int w, double *sum, double *bound)
{
    double acc = 0.0, b = 0.0;
    for (int c = 0; c < p->C; ++c) {
        for (int r = 0; r < p->R; ++r) {
            int y = h * p->stride + r - p->pad;
            if (y < 0 || y >= p->H) continue;
            for (int s = 0; s < p->S; ++s) {
                int x = w * p->stride + s - p->pad;
                if (x < 0 || x >= p->W) continue;
                double wt = Wd[(((int64_t)m * p->C + c) * p->R + r) * p->S + s];
                if (wt == 0.0) continue; /* a zero weight adds nothing to either sum */
                double xi = (double)in[(((int64_t)n * p->C + c) * p->H + y) * p->W + x];
                acc += xi * wt;
                b += fabs(xi * wt);
            }
        }
    }
    *sum = acc;
    *bound = b;
}

static float epilogue(double acc, const float *bias, int m, unsigned flags, double *bound)
{
    if ((flags & ORACLE_F_BIAS) && bias) {
        acc += (double)bias[m];
        *bound += fabs((double)bias[m]);
    }
    if (flags & ORACLE_F_RELU) acc = acc > 0.0 ? acc : 0.0;
    return (float)acc;
}

/* Whole layer: out[N][M][E][F] (fp32) and bound[N][M][E][F] (fp64, sum |w*x| (+|bias|)). */
int oracle_conv(int N, int C, int H, int W, int M, int R, int S, int stride, int pad,
                const float *in, const double *Wd, const float *bias, unsigned flags, float *out,
                double *bound)
{
    shape_t p = {N, C, H, W, M, R, S, stride, pad};
    if (stride < 1 || pad < 0 || H + 2 * pad < R || W + 2 * pad < S) return -1;
    const int E = out_h(&p), F = out_w(&p);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            for (int h = 0; h < E; ++h) {
                for (int w = 0; w < F; ++w) {
                    double acc, b;
                    conv_point(&p, in, Wd, n, m, h, w, &acc, &b);
                    int64_t o = (((int64_t)n * M + m) * E + h) * F + w;
                    out[o] = epilogue(acc, bias, m, flags, &b);
                    if (bound) bound[o] = b;
                }
            }
        }
    }
    return 0;
}

/* Sampled outputs: pts holds npts quadruples (n, m, h, w). */
int oracle_conv_points(int N, int C, int H, int W, int M, int R, int S, int stride, int pad,
                       const float *in, const double *Wd, const float *bias, unsigned flags,
                       int64_t npts, const int32_t *pts, float *out, double *bound)
{
    shape_t p = {N, C, H, W, M, R, S, stride, pad};
    if (stride < 1 || pad < 0 || H + 2 * pad < R || W + 2 * pad < S) return -1;
    const int E = out_h(&p), F = out_w(&p);
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < npts; ++i) {
        int n = pts[4 * i], m = pts[4 * i + 1], h = pts[4 * i + 2], w = pts[4 * i + 3];
        double acc = 0.0, b = 0.0;
        if (n >= 0 && n < N && m >= 0 && m < M && h >= 0 && h < E && w >= 0 && w < F)
            conv_point(&p, in, Wd, n, m, h, w, &acc, &b);
        out[i] = epilogue(acc, bias, m, flags, &b);
        if (bound) bound[i] = b;
    }
    return 0;
}

/* Weight stretching: colidx j -> (c, r, s) -> (c*Hp + r)*Wp + s, Hp/Wp the padded dims. */
int oracle_stretch(int C, int H, int W, int R, int S, int pad, int64_t nnz, const int32_t *colidx,
                   int32_t *stretched)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad;
    for (int64_t j = 0; j < nnz; ++j) {
        int32_t col = colidx[j];
        if (col < 0 || col >= C * R * S) return -1;
        int c = col / (R * S);
        int r = (col / S) % R;
        int s = col % S;
        stretched[j] = (c * Hp + r) * Wp + s;
    }
    return 0;
}

/* Zero-padded input array P[n][c][y+pad][x+pad] = I[n][c][y][x], +0.0f elsewhere. */
int oracle_pad(int N, int C, int H, int W, int pad, const float *in, float *padded)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad;
    for (int64_t i = 0; i < (int64_t)N * C * Hp * Wp; ++i) padded[i] = 0.0f;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x)
                    padded[(((int64_t)n * C + c) * Hp + (y + pad)) * Wp + (x + pad)] =
                        in[(((int64_t)n * C + c) * H + y) * W + x];
    return 0;
}

/* The stretched form of the layer (Section 3.1; the result Algorithm 2 produces): with the
 * padded array P of one image flattened to 1-D, every output element is the sum, over the
 * entries of CSR row m, of value * P[stretched offset + (h*stride)*Wp + w*stride].  Written per
 * output element, like conv_point above but over the row's entries instead of over (c, r, s);
 * fp64 sum.  It must agree with oracle_conv, which pins the padded dims in the offset, the
 * stride on the output coordinate and the per-image pitch C*Hp*Wp. */
int oracle_sconv_alg2(int N, int C, int H, int W, int M, int R, int S, int stride, int pad,
                      const int32_t *rowptr, const int32_t *stretched, const float *value,
                      const float *padded, float *out)
{
    shape_t p = {N, C, H, W, M, R, S, stride, pad};
    const int Wp = W + 2 * pad;
    const int E = out_h(&p), F = out_w(&p);
    const int64_t image_len = (int64_t)C * (H + 2 * pad) * Wp;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            const float *image = padded + n * image_len;
            float *plane = out + ((int64_t)n * M + m) * E * F;
            for (int h = 0; h < E; ++h) {
                for (int w = 0; w < F; ++w) {
                    const int64_t corner = (int64_t)h * stride * Wp + (int64_t)w * stride;
                    double sum = 0.0;
                    for (int32_t e = rowptr[m]; e < rowptr[m + 1]; ++e)
                        sum += (double)value[e] * (double)image[stretched[e] + corner];
                    plane[h * F + w] = (float)sum;
                }
            }
        }
    }
    return 0;
}
