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

namespace {
struct StemShape { int N, C, H, W, K, R, stride, pad, P, Q, taps, kpad; };
int to_stem(const resist_conv_shape *s, StemShape *o) {
  if (!s) return set_error(RESIST_EINVAL, "shape is NULL");
  if (s->dtype != DT_F32 && s->dtype != DT_BF16) return set_error(RESIST_EINVAL, "dtype %d", s->dtype);
  if (s->R != s->S || s->R < 1 || s->stride < 1 || s->pad < 0 || s->N < 1 || s->H < 1 || s->W < 1 || s->C < 1 || s->K < 1)
    return set_error(RESIST_ESHAPE, "stem convolution: bad dimension");
  o->N = s->N; o->C = s->C; o->H = s->H; o->W = s->W; o->K = s->K; o->R = s->R; o->stride = s->stride; o->pad = s->pad;
  o->P = (s->H + 2 * s->pad - s->R) / s->stride + 1;
  o->Q = (s->W + 2 * s->pad - s->R) / s->stride + 1;
  o->taps = s->R * s->R * s->C;
  o->kpad = (o->taps + 31) / 32 * 32;
  if (o->P < 1 || o->Q < 1) return set_error(RESIST_ESHAPE, "empty convolution output");
  const long long lim = 0x7fffffffLL / 4;
  if ((long long)o->N * o->C * o->H * o->W > lim || (long long)o->N * o->P * o->Q * o->K > lim)
    return set_error(RESIST_ESHAPE, "tensor exceeds 2 GiB");
  return RESIST_OK;
}
int64_t stem_partial_floats(const StemShape &g) {
  return stem_wgrad_scratch_floats(g.N, g.C, g.H, g.W, g.K, g.R, g.stride, g.pad, g.P, g.Q, g.kpad);
}
}  // namespace

extern "C" int resist_stem_conv2d_workspace_bytes(const resist_conv_shape *s, int64_t *bytes) {
  StemShape g;
  RESIST_TRY(to_stem(s, &g));
  if (!bytes) return set_error(RESIST_EINVAL, "bytes is NULL");
  const int64_t part = stem_partial_floats(g);
  if (part == 0) return RESIST_ESHAPE;   // message set by the stem's shape check
  *bytes = align256((int64_t)g.K * g.kpad * 4) + align256(part * 4);
  return RESIST_OK;
}

extern "C" int resist_stem_conv2d_forward(const resist_conv_shape *s, const float *x, const float *w, void *y, void *workspace,
                                          int64_t workspace_bytes, void *hip_stream) {
  StemShape g;
  RESIST_TRY(to_stem(s, &g));
  if (!x || !w || !y || !workspace) return set_error(RESIST_EINVAL, "NULL tensor");
  if (workspace_bytes < (int64_t)g.K * g.kpad * 4) return set_error(RESIST_EWORKSPACE, "workspace too small for the padded filter");
  hipStream_t st = (hipStream_t)hip_stream;
  RESIST_TRY(pad_rows(s->dtype, w, workspace, g.K, g.taps, g.kpad, st));
  return stem_conv_fwd(s->dtype, x, workspace, y, nullptr, nullptr, g.N, g.C, g.H, g.W, g.K, g.R, g.stride, g.pad, g.P, g.Q, g.kpad, st);
}

extern "C" int resist_stem_conv2d_wgrad(const resist_conv_shape *s, const void *dy, const float *x, float *dw, void *workspace,
                                        int64_t workspace_bytes, void *hip_stream) {
  StemShape g;
  RESIST_TRY(to_stem(s, &g));
  if (!dy || !x || !dw || !workspace) return set_error(RESIST_EINVAL, "NULL tensor");
  const int64_t part = stem_partial_floats(g);
  if (part == 0) return RESIST_ESHAPE;
  const int64_t pad_bytes = align256((int64_t)g.K * g.kpad * 4);
  if (workspace_bytes < pad_bytes + part * 4) return set_error(RESIST_EWORKSPACE, "workspace too small for the stem weight gradient");
  hipStream_t st = (hipStream_t)hip_stream;
  float *dwpad = (float *)workspace, *partial = (float *)((char *)workspace + pad_bytes);
  RESIST_TRY(stem_conv_wgrad(s->dtype, dy, x, dwpad, partial, g.N, g.C, g.H, g.W, g.K, g.R, g.stride, g.pad, g.P, g.Q, g.kpad, st));
  return unpad_rows_f32(dwpad, dw, g.K, g.taps, g.kpad, st);
}
