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

#ifdef __cplusplus
}
#endif
#endif /* RESIST_OPS_H */
