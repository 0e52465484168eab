/*
 * CPU fp64 oracle for 3x3x3 stride-1 zero-padded 3D convolution on NDHWC volumes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference against which the GPU
 * library is checked.  It shares no code, header or table with the GPU path and
 * must never be called from the product path.
 *
 * What it follows.  The paper (Sec. 2, third paragraph, and Fig. 1) states that a
 * spatially partitioned convolution is: exchange patch margins, pad each patch
 * with what was received, convolve -- and that this is transparent to the user
 * (abstract), i.e. the result is the ordinary convolution of the whole image.
 * The oracle is therefore the plain definition of that ordinary convolution on
 * the unpartitioned volume, written as direct nested loops, with every sum
 * accumulated in double precision in one fixed order (kd, kh, kw, channel).
 * The backward passes (Sec. 3, "Computational efficiency": forward and backward
 * of the convolutions are both on the path) are the exact derivatives of that
 * definition.
 *
 * Conventions (the paper is silent on all of them; these are the build's readings):
 *   - cross-correlation, no tap flip;
 *   - x is zero outside the volume ("same" padding) when pad == 1; with pad == 0
 *     the same loops give the "valid" convolution of an already padded patch;
 *   - layouts: x[N][D][H][W][Cin], w[3][3][3][Cin][Cout], y[N][D][H][W][Cout];
 *   - inputs may be stored as f64, f32 or bf16 bit patterns (dtype codes 0,1,2);
 *     each is widened exactly to double before use; weights, bias and all outputs
 *     are double.
 *
 * Outputs are produced for a caller-chosen sub-box [d0,d1) x [h0,h1) x [w0,w1)
 * so that very large volumes can be checked on samples.
 */
#include <stdint.h>
#include <string.h>
#include <stddef.h>

enum { ORC_F64 = 0, ORC_F32 = 1, ORC_BF16 = 2 };

static inline double ld(const void *p, int dt, size_t i)
{
    if (dt == ORC_F64) return ((const double *)p)[i];
    if (dt == ORC_F32) return (double)((const float *)p)[i];
    /* bf16: the upper 16 bits of an IEEE binary32 */
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* value of volume element (n,d,h,w,c) or 0 when (d,h,w) lies outside the volume */
static inline double at(const void *x, int dt, long D, long H, long W, long C,
                        long n, long d, long h, long w, long c)
{
    if (d < 0 || d >= D || h < 0 || h >= H || w < 0 || w >= W) return 0.0;
    return ld(x, dt, ((((size_t)n * D + d) * H + h) * W + w) * C + c);
}

/*
 * Forward:  z[n,d,h,w,co] = bias[co] + sum_{kd,kh,kw} sum_ci
 *                 x[n, d+kd-pad, h+kh-pad, w+kw-pad, ci] * w[kd,kh,kw,ci,co]
 *           y = max(z,0) if relu else z
 * (D,H,W) are the extents of x.  Output voxel coordinates run over the box, which
 * must lie inside [0, D-2+2*pad) etc.  y has shape [N][d1-d0][h1-h0][w1-w0][Cout].
 */
int orc_conv3d_fwd(const void *x, int xdt, const double *w, const double *bias,
                   double *y, long N, long D, long H, long W, long Cin, long Cout,
                   int pad, int relu, const long *box)
{
    const long d0 = box[0], d1 = box[1], h0 = box[2], h1 = box[3], w0 = box[4], w1 = box[5];
    const long OD = D - 2 + 2 * pad, OH = H - 2 + 2 * pad, OW = W - 2 + 2 * pad;
    if (pad != 0 && pad != 1) return -1;
    if (d0 < 0 || d1 > OD || h0 < 0 || h1 > OH || w0 < 0 || w1 > OW) return -2;
    if (d1 < d0 || h1 < h0 || w1 < w0) return -2;
    const long bd = d1 - d0, bh = h1 - h0, bw = w1 - w0;
    const long rows = N * bd * bh;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        const long n = r / (bd * bh), d = d0 + (r / bh) % bd, h = h0 + r % bh;
        for (long ww = w0; ww < w1; ++ww) {
            double *out = y + ((size_t)r * bw + (ww - w0)) * Cout;
            for (long co = 0; co < Cout; ++co) {
                double acc = bias ? bias[co] : 0.0;
                for (long kd = 0; kd < 3; ++kd)
                    for (long kh = 0; kh < 3; ++kh)
                        for (long kw = 0; kw < 3; ++kw)
                            for (long ci = 0; ci < Cin; ++ci)
                                acc += at(x, xdt, D, H, W, Cin, n, d + kd - pad, h + kh - pad,
                                          ww + kw - pad, ci) *
                                       w[(((kd * 3 + kh) * 3 + kw) * Cin + ci) * Cout + co];
                out[co] = (relu && acc < 0.0) ? 0.0 : acc;
            }
        }
    }
    return 0;
}

/*
 * Data gradient of the 'same' (pad = 1) forward:
 *   dx[n,d,h,w,ci] = sum_{kd,kh,kw} sum_co
 *                 dz[n, d-kd+1, h-kh+1, w-kw+1, co] * w[kd,kh,kw,ci,co]      (dz = 0 outside)
 * (D,H,W) are the extents of dz (= extents of x).  dx has shape [N][box][Cin].
 */
int orc_conv3d_dgrad(const void *dz, int zdt, const double *w, double *dx,
                     long N, long D, long H, long W, long Cin, long Cout, const long *box)
{
    const long d0 = box[0], d1 = box[1], h0 = box[2], h1 = box[3], w0 = box[4], w1 = box[5];
    if (d0 < 0 || d1 > D || h0 < 0 || h1 > H || w0 < 0 || w1 > W) return -2;
    if (d1 < d0 || h1 < h0 || w1 < w0) return -2;
    const long bd = d1 - d0, bh = h1 - h0, bw = w1 - w0;
    const long rows = N * bd * bh;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        const long n = r / (bd * bh), d = d0 + (r / bh) % bd, h = h0 + r % bh;
        for (long ww = w0; ww < w1; ++ww) {
            double *out = dx + ((size_t)r * bw + (ww - w0)) * Cin;
            for (long ci = 0; ci < Cin; ++ci) {
                double acc = 0.0;
                for (long kd = 0; kd < 3; ++kd)
                    for (long kh = 0; kh < 3; ++kh)
                        for (long kw = 0; kw < 3; ++kw)
                            for (long co = 0; co < Cout; ++co)
                                acc += at(dz, zdt, D, H, W, Cout, n, d - kd + 1, h - kh + 1,
                                          ww - kw + 1, co) *
                                       w[(((kd * 3 + kh) * 3 + kw) * Cin + ci) * Cout + co];
                out[ci] = acc;
            }
        }
    }
    return 0;
}

/*
 * Weight gradient:
 *   dw[kd,kh,kw,ci,co] = sum_{n,d,h,w} x[n, d+kd-pad, h+kh-pad, w+kw-pad, ci] * dz[n,d,h,w,co]
 * (D,H,W) are the extents of dz; x has extents (D+2-2*pad, ...) -- i.e. with pad = 1
 * x is the plain volume (zero outside), with pad = 0 it is an already padded patch.
 * Only the `nsel` entries listed in sel[] (flat indices into [3][3][3][Cin][Cout]) are
 * computed, into out[0..nsel); sel == NULL means all 27*Cin*Cout entries in order.
 * Each entry is one sum in the fixed order n, d, h, w.
 */
int orc_conv3d_wgrad(const void *x, int xdt, const void *dz, int zdt, double *out,
                     long N, long D, long H, long W, long Cin, long Cout, int pad,
                     const long *sel, long nsel)
{
    if (pad != 0 && pad != 1) return -1;
    const long total = 27 * Cin * Cout;
    const long XD = D + 2 - 2 * pad, XH = H + 2 - 2 * pad, XW = W + 2 - 2 * pad;
    const long cnt = sel ? nsel : total;
    for (long i = 0; i < cnt; ++i)
        if (sel && (sel[i] < 0 || sel[i] >= total)) return -2;
#pragma omp parallel for schedule(dynamic, 1)
    for (long i = 0; i < cnt; ++i) {
        const long e = sel ? sel[i] : i;
        const long co = e % Cout, ci = (e / Cout) % Cin, tap = e / (Cout * Cin);
        const long kd = tap / 9, kh = (tap / 3) % 3, kw = tap % 3;
        double acc = 0.0;
        for (long n = 0; n < N; ++n)
            for (long d = 0; d < D; ++d)
                for (long h = 0; h < H; ++h)
                    for (long ww = 0; ww < W; ++ww)
                        acc += at(x, xdt, XD, XH, XW, Cin, n, d + kd - pad, h + kh - pad,
                                  ww + kw - pad, ci) *
                               ld(dz, zdt, ((((size_t)n * D + d) * H + h) * W + ww) * Cout + co);
        out[i] = acc;
    }
    return 0;
}

/* Bias gradient: db[co] = sum over all voxels of dz[.,co], fixed order. */
int orc_bias_grad(const void *dz, int zdt, double *db, long nvox, long Cout)
{
#pragma omp parallel for schedule(static)
    for (long co = 0; co < Cout; ++co) {
        double acc = 0.0;
        for (long v = 0; v < nvox; ++v) acc += ld(dz, zdt, (size_t)v * Cout + co);
        db[co] = acc;
    }
    return 0;
}
