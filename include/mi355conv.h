/*
 * mi355conv — fp32 NHWC 2-D convolution for small feature maps on AMD MI355X (gfx950).
 *
 * C ABI of the three operators that the paper's fp32 GPU library contributes and
 * that its Sec. IV credits for the training speed on 32x32 images: forward
 * convolution, deconvolution (= backward-data) and backward-weight
 * (Sec. III "Layer-1 Native libs"; Sec. IV, paragraph on the small-feature-map
 * conv\deconv operators; Table I: float32, tensors in [N,H,W,C] order; Fig. 2:
 * argument set in_channel, out_channel, kernel, stride, padding).
 *
 * Conventions shared by every entry point
 *   - Tensors are dense fp32, last index fastest, DEVICE pointers, 16-byte aligned:
 *       X, dX : [N, IH, IW, IC]        W, dW : [OC, FH, FW, IC]
 *       Y, dY : [N, OH, OW, OC]        OH = floor((IH + 2*ph - FH)/sh) + 1 (same in w)
 *   - Cross-correlation (no filter flip), zero padding, dilation 1, groups 1, no bias.
 *   - Outputs are overwritten (beta = 0) and every element is written, including the
 *     zeros of dX that no filter tap reaches.  Inputs are never modified.  Input and
 *     output must not alias.
 *   - The caller owns all memory, including the workspace.  The library allocates no
 *     device memory and keeps no pointer after returning.
 *   - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and return; completion is the caller's stream synchronisation
 *     (the paper's async mode, Sec. III Layer-4).  Calls on different streams are safe
 *     if their outputs and workspaces do not overlap.
 *   - Every tensor must hold fewer than 2^31 elements.
 *   - All argument checks happen before the first HIP call, so they can be exercised
 *     on a machine without a GPU.
 *   - Return value: MI355CONV_OK (0) or a negative mi355conv_status.
 *   - Stream capture: the operator entry points only enqueue kernels (no allocation, no
 *     memset, no synchronisation), so they may be recorded into a HIP graph.  The first
 *     operator call on a device also does one-time device set-up (kernel attributes, address
 *     look-up), which must not happen inside a capture: call conv2d_init() - or any operator
 *     once - on that device before capturing.
 *   - Process-global tuning: conv2d_set_tuning / conv2d_set_tile change what
 *     conv2d_workspace_bytes, conv2d_query_plan, conv2d_query_workgroup and every operator
 *     entry point choose from then on, in all threads.  They exist for tests and sweeps; a
 *     program that calls operators from several threads or streams leaves them alone (or sets
 *     them once before it starts), because a workspace sized under one tuning may be too small
 *     under another (the entry point then returns MI355CONV_ERR_WORKSPACE, it never overruns).
 */
#ifndef MI355CONV_H
#define MI355CONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mi355conv_status {
    MI355CONV_OK = 0,
    MI355CONV_ERR_NULL_PTR = -1,    /* a required pointer is NULL                          */
    MI355CONV_ERR_BAD_DIM = -2,     /* dim <= 0, stride <= 0, pad < 0, OH/OW <= 0, >= 2^31 */
    MI355CONV_ERR_WORKSPACE = -3,   /* ws_bytes below conv2d_workspace_bytes(), or ws NULL */
    MI355CONV_ERR_ALIGNMENT = -4,   /* a tensor or the workspace is not 16-byte aligned    */
    MI355CONV_ERR_UNSUPPORTED = -5, /* bad op code / tuning value / shape an entry point does not take */
    MI355CONV_ERR_HIP = -6          /* a HIP runtime call or kernel launch failed          */
} mi355conv_status;

/* Operator codes for conv2d_workspace_bytes / conv2d_query_plan. */
enum { MI355CONV_OP_FWD = 0, MI355CONV_OP_BWD_DATA = 1, MI355CONV_OP_BWD_WEIGHT = 2 };

/* Problem shape.  Square configurations set sh == sw and ph == pw. */
typedef struct conv2d_desc {
    int N, IH, IW, IC;   /* input batch, height, width, channels */
    int OC, FH, FW;      /* output channels, filter height, width */
    int sh, sw;          /* stride (>= 1) */
    int ph, pw;          /* symmetric zero padding (>= 0) */
} conv2d_desc;

/* Kernel variants (conv2d_plan_info.variant, conv2d_set_tuning). */
enum {
    MI355CONV_VARIANT_AUTO = -1,
    MI355CONV_VARIANT_DIRECT = 0,  /* one thread per output element; any shape             */
    MI355CONV_VARIANT_MFMA = 1     /* implicit GEMM on v_mfma_f32_32x32x2_f32, LDS-staged  */
};

/* What the host-side selection picked for a problem (the paper's "operators selected by a
 * feature-map-size threshold", Sec. IV; Sec. III Layer-2 holds that logic). */
typedef struct conv2d_plan_info {
    int variant;        /* MI355CONV_VARIANT_*                                              */
    int tile_m, tile_n; /* workgroup output tile (GEMM rows x cols); 0 for DIRECT           */
    int split;          /* number of reduction slices (1 = no split)                        */
    int pos_major;      /* 1: GEMM rows ordered (oh,ow,n) so tiles skip padded taps         */
    int grid;           /* workgroups of the main kernel                                    */
    size_t workspace_bytes;
    int kernel;         /* MI355CONV_KERNEL_*: which kernel family runs the plan            */
    int order;          /* MI355CONV_ORDER_*: how workgroup ids map to tiles                */
} conv2d_plan_info;

/* Workgroup orders (conv2d_plan_info.order). */
enum {
    MI355CONV_ORDER_PLAIN = 0,     /* tiles in id order (ids regrouped so that neighbours share an XCD) */
    MI355CONV_ORDER_LONGEST = 1,   /* unequal tiles dealt longest first to the 256 CUs                 */
    MI355CONV_ORDER_REGIONS = 2    /* every XCD owns a part of the tiles that shares operands          */
};

/* Kernel families (conv2d_plan_info.kernel); for tests, which force every compiled variant. */
enum {
    MI355CONV_KERNEL_DIRECT = 0,
    MI355CONV_KERNEL_GATHER = 1,       /* gather-GEMM, 16-byte loads along the channel axis     */
    MI355CONV_KERNEL_GATHER_ELEM = 2,  /* gather-GEMM, element-wise loads (any channel count)   */
    MI355CONV_KERNEL_FIRST_LAYER = 3,  /* the kernels for at most 32 patch columns / 4 channels */
    MI355CONV_KERNEL_WGRAD = 4,        /* backward-weight, any map shape                        */
    MI355CONV_KERNEL_WGRAD_FAST = 5    /* backward-weight, aligned maps                         */
};

/* One-time set-up of the CURRENT device (idempotent, thread-safe): raises the LDS limit of the
 * large-tile kernels and looks up the library's own device memory.  Optional - the first operator
 * call on a device does the same - except before stream capture, where it (or one operator call)
 * is required.  Must not be called while a capture is under way. */
int conv2d_init(void);

/* Bytes of device workspace the given operator needs for this shape under the current
 * tuning (0 is possible).  Returns 0 on invalid arguments too; the entry points report
 * the error. */
size_t conv2d_workspace_bytes(int op, const conv2d_desc *d);

/* Fill *info with the plan the entry point would run.  Host only; no HIP call. */
int conv2d_query_plan(int op, const conv2d_desc *d, conv2d_plan_info *info);

/* Where the plan would send hardware workgroup id `workgroup` (0 <= workgroup < grid): its
 * rank in the order "longest work first" and the relative length of that work item (taps or
 * live positions; 1 for plans whose workgroups are all alike).  While a launch is resident,
 * workgroup ids 256 apart share a CU; the library deals unequal work items to the CUs through
 * this mapping (paper Sec. IV: the small-feature-map operators).  Host only; for tests. */
int conv2d_query_workgroup(int op, const conv2d_desc *d, int workgroup, int *rank, int *work);

/* The tile that workgroup id `workgroup` of a region-wise / group-wise launch
 * (conv2d_plan_info.order == MI355CONV_ORDER_REGIONS) works on: its row tile (forward /
 * backward-data: tile_m rows of the GEMM in (y,x,n) order; backward-weight: tile_m output
 * channels), column tile and reduction slice - computed by the functions the kernels use.
 * MI355CONV_ERR_UNSUPPORTED for the other orders.  Host only; for tests, which check that the
 * ids of a launch map one-to-one onto its tiles. */
int conv2d_query_tile(int op, const conv2d_desc *d, int workgroup, int *row_tile, int *col_tile, int *slice);

/* Process-wide override for tests and sweeps: variant = MI355CONV_VARIANT_AUTO or a
 * variant code, split = 0 (auto) or a forced slice count >= 1 (clamped to what the shape
 * allows).  Not thread-safe against concurrent operator calls. */
int conv2d_set_tuning(int variant, int split);

/* Second process-wide override for sweeps: workgroup tile of the MFMA variants
 * (tile_m x tile_n must be a compiled pair, 0 x 0 = auto) and the row order
 * (pos_major = -1 auto, 0 (n,y,x) rows, 1 (y,x,n) rows where the shape allows it). */
int conv2d_set_tile(int tile_m, int tile_n, int pos_major);

/* Third process-wide override for tests and sweeps: the order in which the workgroups of a
 * launch with (y,x,n) rows (forward, unit-stride backward-data, backward-weight on small maps)
 * are dealt to the chip.  region_wise = 1 (default): every XCD (workgroup id modulo 8, one L2
 * each) owns a part of the tiles that shares operands - a spatial region x image group x
 * filter-slice group for the gather operators, a group of output-channel tiles x
 * input-channel tiles x slices for backward-weight - wherever the shape allows it; 0: the
 * older order (longest tiles first over the whole chip).  Results are bitwise equal either
 * way. */
int conv2d_set_order(int region_wise);

/* Forward convolution (Sec. III Layer-1; Fig. 2 conv3D arguments):
 *   Y[n,oh,ow,oc] = sum_{fh,fw,ic} X[n, oh*sh-ph+fh, ow*sw-pw+fw, ic] * W[oc,fh,fw,ic],
 * X taken as 0 outside the image.  X, W: device, read-only.  Y: device, overwritten.
 * ws: device scratch of at least conv2d_workspace_bytes(OP_FWD, d) bytes (may be NULL
 * when that is 0). */
int conv2d_fwd(const float *X, const float *W, float *Y, const conv2d_desc *d,
               void *ws, size_t ws_bytes, void *stream);

/* Forward convolution with the bias add and the leaky-ReLU activation of the paper's layer
 * constructors (Fig. 2: conv3D(..., biased), leakyRelu) applied in the kernel's epilogue:
 *   Y[n,oh,ow,oc] = act(conv(X,W)[n,oh,ow,oc] + bias[oc]),  act(v) = v > 0 ? v : negative_slope * v.
 * bias: device pointer to OC floats, or NULL for no bias; negative_slope = 1 means no
 * activation, 0 is ReLU.  Everything else (layouts, workspace, errors, enqueue-only) as
 * conv2d_fwd; when the reduction is sliced the epilogue runs in the combine pass. */
int conv2d_fwd_bias_act(const float *X, const float *W, const float *bias, float *Y,
                        const conv2d_desc *d, float negative_slope, void *ws, size_t ws_bytes,
                        void *stream);

/* First-layer forward from 8-bit pixels: X8 holds unsigned bytes [N,IH,IW,IC] (device); every
 * pixel is converted on load, x = (float)byte * scale (the paper converts pixel bytes to floats
 * on the device, Sec. III; Table I scales by 1/255), then as conv2d_fwd.  X8 needs no alignment.
 * Only shapes the first-layer kernel takes (FH*FW*IC <= 32, and IC <= 4 or not a multiple of 4),
 * under automatic tuning; MI355CONV_ERR_UNSUPPORTED otherwise.  No workspace. */
int conv2d_fwd_u8(const unsigned char *X8, float scale, const float *W, float *Y,
                  const conv2d_desc *d, void *stream);

/* Backward-data = deconvolution (Sec. IV: the deconv operator for small feature maps):
 *   dX[n,ih,iw,ic] = sum over (oc,fh,fw) with oh*sh-ph+fh == ih, ow*sw-pw+fw == iw of
 *                    dY[n,oh,ow,oc] * W[oc,fh,fw,ic].
 * d->IH, d->IW give the size of dX (the transposed convolution's output size is not
 * unique when (IH+2ph-FH) % sh != 0); elements no tap reaches are written as 0.
 * deconv2d is the same function under the paper's name for it. */
int conv2d_bwd_data(const float *dY, const float *W, float *dX, const conv2d_desc *d,
                    void *ws, size_t ws_bytes, void *stream);
int deconv2d(const float *dY, const float *W, float *dX, const conv2d_desc *d,
             void *ws, size_t ws_bytes, void *stream);

/* Backward-weight (implied by the paper's training loop, Fig. 2 backward + update):
 *   dW[oc,fh,fw,ic] = sum_{n,oh,ow} dY[n,oh,ow,oc] * X[n, oh*sh-ph+fh, ow*sw-pw+fw, ic]
 * over in-range taps.  Unless the output alone fills the chip, the sum over N*OH*OW is cut
 * into slices whose partial results go through the workspace and are combined in a fixed
 * order, so results are bitwise reproducible either way. */
int conv2d_bwd_weight(const float *X, const float *dY, float *dW, const conv2d_desc *d,
                      void *ws, size_t ws_bytes, void *stream);

/* Backward-weight for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operator,
 * same plan and same kernels as conv2d_bwd_weight; the slice partials go to a device array that is
 * part of the library (conv2d_noalloc_scratch_bytes() bytes, 32 MiB, held by every GPU the library
 * runs on until the process ends) instead of a caller workspace.  The call allocates nothing and
 * frees nothing.  Returns MI355CONV_ERR_WORKSPACE, before any HIP call, when the shape needs more
 * than that (conv2d_workspace_bytes(MI355CONV_OP_BWD_WEIGHT, d) tells).  All calls on one GPU share
 * that GPU's array: two such calls that may run at the same time on one GPU (different streams)
 * race; calls on one stream are ordered and safe.  Nothing in the array needs clearing between
 * calls (every partial that is read was written by the same call).  As with every operator, the
 * first call on a device must not be inside a stream capture (conv2d_init). */
int conv2d_bwd_weight_noalloc(const float *X, const float *dY, float *dW, const conv2d_desc *d,
                              void *stream);
size_t conv2d_noalloc_scratch_bytes(void);

/* Matrix multiply of the paper's fully-connected layer (Fig. 2 fullconnect; Sec. II names the
 * operator family matMul / matMulT1), served by the 1x1 operators on a 1x1 map - dense fp32
 * row-major matrices, device pointers, 16-byte aligned, C overwritten:
 *   MI355CONV_MATMUL_NT  C[M,N] = A[M,K] * B[N,K]^T    the layer's forward      Y  = X  W^T
 *   MI355CONV_MATMUL_NN  C[M,N] = A[M,K] * B[K,N]      its input gradient       dX = dY W
 *   MI355CONV_MATMUL_TN  C[M,N] = A[K,M]^T * B[K,N]    its weight gradient      dW = dY^T X
 * Workspace, stream, errors and enqueue-only behaviour as for the convolution entry points;
 * matmul_workspace_bytes gives the workspace size (0 on invalid arguments). */
enum { MI355CONV_MATMUL_NT = 0, MI355CONV_MATMUL_NN = 1, MI355CONV_MATMUL_TN = 2 };
size_t matmul_workspace_bytes(int kind, int M, int N, int K);
int matmul_f32(int kind, const float *A, const float *B, float *C, int M, int N, int K,
               void *ws, size_t ws_bytes, void *stream);

/* Measurement aid (not an operator): launches a register-only v_mfma_f32_32x32x2_f32 loop with
 * valu_per_8_mfma in {0, 16, 48, 96} ordinary vector instructions per 8 matrix instructions, on
 * `workgroups` workgroups of 256 threads, `iters` x 8 matrix instructions per wave, i.e.
 * workgroups * 4 * iters * 8 * 4096 FLOP.  out: device, workgroups * 256 floats (written so the
 * loop is not optimised away).  The caller times the launch; bench.py --mfma-peak reports the
 * sustained fp32 matrix rate that the "% of measured peak" figures refer to. */
int conv2d_probe_mfma_rate(int valu_per_8_mfma, int workgroups, int iters, float *out, void *stream);

/* Static text for a status code. */
const char *conv2d_status_string(int status);

/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char *conv2d_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MI355CONV_H */
