/*
 * resist_ops.h -- layer-level entry points of the same library: the convolution kernels that
 * resist_local_step is built from, exposed so each can be checked against the textbook
 * definition on its own.  Same conventions as resist.h (status codes, caller-owned device
 * memory, caller's stream, no synchronisation).
 *
 * Layouts: activations NHWC [N][H][W][C]; filters [K][R][S][C]; outputs [N][P][Q][K] with
 * P = (H + 2*pad - R)/stride + 1.  dtype 0: all fp32.  dtype 1: activations and filters bf16
 * (as uint16 bit patterns), accumulation fp32, weight gradients fp32.
 * Supported: R = S in {1,3,5,7}; stride in {1,2}; 0 <= pad < R; C and K multiples of 4 (fp32) or 8
 * (bf16); the stride-2 data gradient needs even H and W; every tensor below 2 GiB.  Anything else is
 * RESIST_ESHAPE before any launch.
 */
#ifndef RESIST_OPS_H
#define RESIST_OPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t N, H, W, C; /* input activation */
  int32_t K, R, S;    /* filter           */
  int32_t stride, pad;
  int32_t dtype;      /* 0 fp32, 1 bf16   */
} resist_conv_shape;

/* Workspace (bytes) the three calls below need at most for this shape.  host. */
int resist_conv2d_workspace_bytes(const resist_conv_shape *s, int64_t *bytes);

/* y[n,p,q,k] = sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[k,r,s,c]  (zero padding) */
int resist_conv2d_forward(const resist_conv_shape *s, const void *x, const void *w, void *y,
                          void *workspace, int64_t workspace_bytes, void *hip_stream);

/* dx[n,h,w,c] = sum over (k,r,s,p,q) with h = p*stride+r-pad, w = q*stride+s-pad of
 * dy[n,p,q,k] * w[k,r,s,c] */
int resist_conv2d_dgrad(const resist_conv_shape *s, const void *dy, const void *w, void *dx,
                        void *workspace, int64_t workspace_bytes, void *hip_stream);

/* dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride+r-pad, q*stride+s-pad, c]; dw is fp32 */
int resist_conv2d_wgrad(const resist_conv_shape *s, const void *dy, const void *x, float *dw,
                        void *workspace, int64_t workspace_bytes, void *hip_stream);

/*
 * The stem convolution: the first layer reads the input batch as the caller passes it to
 * resist_local_step -- logical [N,C,H,W] fp32 with C <= 4 -- and runs as an implicit GEMM over the
 * R*S*C filter positions (no im2col matrix is written).  The resist_conv_shape describes the same
 * convolution (N, H, W, C of the image; K, R = S, stride, pad; dtype of the OUTPUT side: 0 fp32, 1 bf16,
 * in which case image and filter are rounded to bf16 as they become matrix operands).
 * Supported: C <= 4, K a multiple of 16 up to 128, R*S*C <= 160, tensors below 2 GiB.
 *   x   device [N][C][H][W] fp32           w   device [K][R][S][C] fp32 (the master filter)
 *   y   device [N][P][Q][K] in dtype       dy  device [N][P][Q][K] in dtype      dw  device [K][R][S][C] fp32
 * Workspace: resist_stem_conv2d_workspace_bytes (padded filter copies and the partial sums of the
 * weight gradient).
 */
int resist_stem_conv2d_workspace_bytes(const resist_conv_shape *s, int64_t *bytes);
int resist_stem_conv2d_forward(const resist_conv_shape *s, const float *x, const float *w, void *y, void *workspace,
                               int64_t workspace_bytes, void *hip_stream);
int resist_stem_conv2d_wgrad(const resist_conv_shape *s, const void *dy, const float *x, float *dw, void *workspace,
                             int64_t workspace_bytes, void *hip_stream);

/*
 * resist_conv2d_wgrad for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same
 * bits as resist_conv2d_wgrad, but the split partial sums go to a static device array inside the
 * library (32 MiB per GPU, held until the process ends; resist_conv2d_wgrad_static_limit reports the
 * size).  The call allocates nothing (keep resist_profile_enable off: timing creates events).
 * RESIST_EWORKSPACE if the shape's partial sums (resist_conv2d_workspace_bytes' split part) exceed
 * the array.  Nothing in the array needs clearing between calls: every split writes its whole slice
 * before the reduction reads it.  All calls on one GPU share the array, so two calls that overlap in
 * time on one GPU (different streams, or different host threads) race; calls on one stream do not.
 */
int resist_conv2d_wgrad_static(const resist_conv_shape *s, const void *dy, const void *x, float *dw,
                               void *hip_stream);
int resist_conv2d_wgrad_static_limit(int64_t *bytes);

#ifdef __cplusplus
}
#endif
#endif /* RESIST_OPS_H */
