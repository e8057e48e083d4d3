/*
 * CPU oracle for fp32 NHWC 2-D convolution and its two adjoints.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path and the product never calls it.
 *
 * The paper (Sec. III "Layer-1 Native libs", Sec. IV discussion of the
 * small-feature-map conv\deconv operators, Table I: float32, [N,H,W,C]
 * order) names the operators but prints no formula; they are the standard
 * deep-learning cross-correlation and its adjoints:
 *
 *   fwd        Y[n,oh,ow,oc]  = sum_{fh,fw,ic} X[n, oh*sh-ph+fh, ow*sw-pw+fw, ic] * W[oc,fh,fw,ic]
 *   bwd_data   dX[n,ih,iw,ic] = sum_{oc,fh,fw} G[n,oh,ow,oc] * W[oc,fh,fw,ic]
 *                               over (fh,fw) with oh*sh-ph+fh == ih, ow*sw-pw+fw == iw
 *   bwd_weight dW[oc,fh,fw,ic]= sum_{n,oh,ow}  G[n,oh,ow,oc] * X[n, oh*sh-ph+fh, ow*sw-pw+fw, ic]
 *
 * with X zero outside [0,IH)x[0,IW), OH = floor((IH+2ph-FH)/sh)+1 (same
 * in w).  Layouts: X,dX [N,IH,IW,IC]; W,dW [OC,FH,FW,IC]; Y,G [N,OH,OW,OC];
 * dense, last index fastest.  Inputs are fp32; every product and every sum
 * is taken in fp64 and the result is returned in fp64 (the caller rounds).
 *
 * Each routine is the literal loop nest: one accumulator per output
 * element, summed in the order the loops run.  OpenMP splits only the
 * outermost output index, so no accumulator is shared between threads and
 * the result does not depend on the thread count.
 */
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_extent(int in, int pad, int f, int stride)
{
    int span = in + 2 * pad - f;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* Y[n,oh,ow,oc]: loops n, oh, ow, oc, fh, fw, ic. */
void oracle_conv2d_fwd(const float *X, const float *W, double *Y,
                       int N, int IH, int IW, int IC, int OC,
                       int FH, int FW, int sh, int sw, int ph, int pw)
{
    const int OH = out_extent(IH, ph, FH, sh);
    const int OW = out_extent(IW, pw, FW, sw);
    i64 rows = (i64)N * OH;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < rows; ++r) {
        int n = (int)(r / OH), oh = (int)(r % OH);
        for (int ow = 0; ow < OW; ++ow)
            for (int oc = 0; oc < OC; ++oc) {
                double acc = 0.0;
                for (int fh = 0; fh < FH; ++fh) {
                    int ih = oh * sh - ph + fh;
                    if (ih < 0 || ih >= IH) continue;
                    for (int fw = 0; fw < FW; ++fw) {
                        int iw = ow * sw - pw + fw;
                        if (iw < 0 || iw >= IW) continue;
                        const float *x = X + (((i64)n * IH + ih) * IW + iw) * IC;
                        const float *w = W + (((i64)oc * FH + fh) * FW + fw) * IC;
                        for (int ic = 0; ic < IC; ++ic)
                            acc += (double)x[ic] * (double)w[ic];
                    }
                }
                Y[(((i64)n * OH + oh) * OW + ow) * OC + oc] = acc;
            }
    }
}

/* dX[n,ih,iw,ic]: gather form, loops n, ih, iw, ic, fh, fw, oc.
 * A tap (fh,fw) contributes iff ih+ph-fh is a non-negative multiple of sh
 * whose quotient is a valid oh (same in w).  Elements no tap reaches are 0. */
void oracle_conv2d_bwd_data(const float *G, const float *W, double *dX,
                            int N, int IH, int IW, int IC, int OC,
                            int FH, int FW, int sh, int sw, int ph, int pw)
{
    const int OH = out_extent(IH, ph, FH, sh);
    const int OW = out_extent(IW, pw, FW, sw);
    i64 rows = (i64)N * IH;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < rows; ++r) {
        int n = (int)(r / IH), ih = (int)(r % IH);
        for (int iw = 0; iw < IW; ++iw)
            for (int ic = 0; ic < IC; ++ic) {
                double acc = 0.0;
                for (int fh = 0; fh < FH; ++fh) {
                    int th = ih + ph - fh;
                    if (th < 0 || th % sh != 0) continue;
                    int oh = th / sh;
                    if (oh >= OH) continue;
                    for (int fw = 0; fw < FW; ++fw) {
                        int tw = iw + pw - fw;
                        if (tw < 0 || tw % sw != 0) continue;
                        int ow = tw / sw;
                        if (ow >= OW) continue;
                        const float *g = G + (((i64)n * OH + oh) * OW + ow) * OC;
                        for (int oc = 0; oc < OC; ++oc)
                            acc += (double)g[oc] *
                                   (double)W[(((i64)oc * FH + fh) * FW + fw) * IC + ic];
                    }
                }
                dX[(((i64)n * IH + ih) * IW + iw) * IC + ic] = acc;
            }
    }
}

/* dW[oc,fh,fw,ic]: loops oc, fh, fw, ic, n, oh, ow. */
void oracle_conv2d_bwd_weight(const float *X, const float *G, double *dW,
                              int N, int IH, int IW, int IC, int OC,
                              int FH, int FW, int sh, int sw, int ph, int pw)
{
    const int OH = out_extent(IH, ph, FH, sh);
    const int OW = out_extent(IW, pw, FW, sw);
    i64 rows = (i64)OC * FH;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < rows; ++r) {
        int oc = (int)(r / FH), fh = (int)(r % FH);
        for (int fw = 0; fw < FW; ++fw)
            for (int ic = 0; ic < IC; ++ic) {
                double acc = 0.0;
                for (int n = 0; n < N; ++n)
                    for (int oh = 0; oh < OH; ++oh) {
                        int ih = oh * sh - ph + fh;
                        if (ih < 0 || ih >= IH) continue;
                        for (int ow = 0; ow < OW; ++ow) {
                            int iw = ow * sw - pw + fw;
                            if (iw < 0 || iw >= IW) continue;
                            acc += (double)G[(((i64)n * OH + oh) * OW + ow) * OC + oc] *
                                   (double)X[(((i64)n * IH + ih) * IW + iw) * IC + ic];
                        }
                    }
                dW[(((i64)oc * FH + fh) * FW + fw) * IC + ic] = acc;
            }
    }
}

/* Matrix multiply of the paper's fully-connected layer (Fig. 2 fullconnect; Sec. II names the
 * operator family matMul / matMulT1): C[M,N] = op(A) * op(B) in fp64, row-major operands,
 *   ta == 0: op(A)[i,k] = A[i*K + k]  (A is M x K)      ta != 0: op(A)[i,k] = A[k*M + i]  (A is K x M)
 *   tb == 0: op(B)[k,j] = B[k*N + j]  (B is K x N)      tb != 0: op(B)[k,j] = B[j*K + k]  (B is N x K)
 * One accumulator per output element, the definition written out. */
void oracle_matmul(const float *A, const float *B, double *C, int M, int N, int K, int ta, int tb)
{
#pragma omp parallel for schedule(static)
    for (i64 i = 0; i < M; ++i)
        for (int j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                const double a = ta ? (double)A[(i64)k * M + i] : (double)A[i * K + k];
                const double b = tb ? (double)B[(i64)j * K + k] : (double)B[(i64)k * N + j];
                acc += a * b;
            }
            C[i * N + j] = acc;
        }
}
