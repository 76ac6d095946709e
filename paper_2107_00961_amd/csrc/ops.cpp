// Layer-level C entry points (resist_ops.h): the convolution kernels on their own.
#include "internal.h"

using namespace resist;

namespace {
int to_geom(const resist_conv_shape *s, ConvGeom *g) {
  if (!s) return set_error(RESIST_EINVAL, "shape is NULL");
  if (s->dtype != DT_F32 && s->dtype != DT_BF16) return set_error(RESIST_EINVAL, "dtype %d", s->dtype);
  if (s->R != s->S) return set_error(RESIST_ESHAPE, "only square filters");
  if (s->N < 1 || s->H < 1 || s->W < 1 || s->C < 1 || s->K < 1 || s->R < 1 || s->stride < 1 || s->pad < 0)
    return set_error(RESIST_ESHAPE, "non-positive dimension");
  *g = make_geom(s->N, s->H, s->W, s->C, s->K, s->R, s->stride, s->pad);
  return RESIST_OK;
}
int64_t align256(int64_t b) { return (b + 255) & ~(int64_t)255; }
}  // namespace

extern "C" int resist_conv2d_workspace_bytes(const resist_conv_shape *s, int64_t *bytes) {
  ConvGeom g;
  RESIST_TRY(to_geom(s, &g));
  if (!bytes) return set_error(RESIST_EINVAL, "bytes is NULL");
  const int64_t filt = align256((int64_t)g.K * g.R * g.S * g.C * esize(s->dtype));
  const int64_t split = align256(wgrad_scratch_floats(g) * 4);
  *bytes = std::max<int64_t>(std::max(filt, split), 256);
  return RESIST_OK;
}

extern "C" int resist_conv2d_forward(const resist_conv_shape *s, const void *x, const void *w, void *y, void *workspace,
                                     int64_t workspace_bytes, void *hip_stream) {
  ConvGeom g;
  RESIST_TRY(to_geom(s, &g));
  if (!x || !w || !y) return set_error(RESIST_EINVAL, "NULL tensor");
  (void)workspace; (void)workspace_bytes;
  return conv_fwd(g, s->dtype, x, w, y, nullptr, nullptr, nullptr, (hipStream_t)hip_stream);
}

extern "C" int resist_conv2d_dgrad(const resist_conv_shape *s, const void *dy, const void *w, void *dx, void *workspace,
                                   int64_t workspace_bytes, void *hip_stream) {
  ConvGeom g;
  RESIST_TRY(to_geom(s, &g));
  if (!dy || !w || !dx || !workspace) return set_error(RESIST_EINVAL, "NULL tensor");
  if (workspace_bytes < (int64_t)g.K * g.R * g.S * g.C * esize(s->dtype)) return set_error(RESIST_EWORKSPACE, "workspace too small for the transposed filter");
  hipStream_t st = (hipStream_t)hip_stream;
  RESIST_TRY(prepare_filter(g, s->dtype, s->dtype, w, nullptr, workspace, st));
  return conv_dgrad(g, s->dtype, dy, workspace, dx, nullptr, nullptr, st);
}

extern "C" int resist_conv2d_wgrad(const resist_conv_shape *s, const void *dy, const void *x, float *dw, void *workspace,
                                   int64_t workspace_bytes, void *hip_stream) {
  ConvGeom g;
  RESIST_TRY(to_geom(s, &g));
  if (!dy || !x || !dw) return set_error(RESIST_EINVAL, "NULL tensor");
  const int64_t need = wgrad_scratch_floats(g) * 4;
  if (need > 0 && (!workspace || workspace_bytes < need)) return set_error(RESIST_EWORKSPACE, "workspace too small for split-K partial sums");
  return conv_wgrad(g, s->dtype, dy, x, dw, (float *)workspace, (hipStream_t)hip_stream);
}

extern "C" int resist_conv2d_wgrad_static(const resist_conv_shape *s, const void *dy, const void *x, float *dw, void *hip_stream) {
  ConvGeom g;
  RESIST_TRY(to_geom(s, &g));
  if (!dy || !x || !dw) return set_error(RESIST_EINVAL, "NULL tensor");
  return conv_wgrad_static(g, s->dtype, dy, x, dw, (hipStream_t)hip_stream);
}

extern "C" int resist_conv2d_wgrad_static_limit(int64_t *bytes) {
  if (!bytes) return set_error(RESIST_EINVAL, "bytes is NULL");
  *bytes = wgrad_static_scratch_bytes();
  return RESIST_OK;
}
