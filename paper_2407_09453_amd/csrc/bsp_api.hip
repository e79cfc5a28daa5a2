// extern "C" device entry points: argument checks, shape arithmetic, dispatch.
#include "bsp.h"
#include "bsp_launch.h"

#include <limits>

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int prepare(const bsp_weights* w, const void* X, const float* bias, void* Y, int32_t B,
            int32_t L, int32_t J, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
            ConvParams* out, bool integer = false) {
  if (!w || (B != 0 && (!X || !Y))) return BSP_ERR_NULL;  // an empty batch needs no X or Y
  if (!w->plan || !w->plan_host) return BSP_ERR_NULL;
  if (w->nnzb > 0 && !w->payload) return BSP_ERR_NULL;
  if (w->O <= 0 || w->I <= 0 || w->H <= 0 || w->K <= 0 || w->nnzb < 0) return BSP_ERR_SHAPE;
  if (!((w->bo == 8 && w->bi == 8) || (w->bo == 4 && w->bi == 16) || (w->bo == 16 && w->bi == 4)))
    return BSP_ERR_UNSUPPORTED;
  if (integer ? w->dtype != BSP_I8 : (w->dtype != BSP_F32 && w->dtype != BSP_BF16))
    return BSP_ERR_DTYPE;
  if (B < 0 || L <= 0 || J <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return BSP_ERR_SHAPE;
  if (L + 2 * (int64_t)ph < w->H || J + 2 * (int64_t)pw < w->K) return BSP_ERR_SHAPE;
  const int64_t M = (L + 2 * (int64_t)ph - w->H) / sh + 1;
  const int64_t N = (J + 2 * (int64_t)pw - w->K) / sw + 1;
  if (M < 1 || N < 1) return BSP_ERR_SHAPE;
  const int64_t lim = std::numeric_limits<int32_t>::max();
  if ((int64_t)B * M * N > lim || (int64_t)B * M * N * w->O > lim * 4 ||
      (int64_t)B * L * J * w->I > lim * 4)
    return BSP_ERR_SHAPE;
  if (w->plan_bytes < (int64_t)BSP_PLAN_HEADER_WORDS * 4) return BSP_ERR_CAPACITY;
  if ((B != 0 && ((integer ? (reinterpret_cast<uintptr_t>(X) & 7u) != 0 : !aligned16(X)) ||
                  !aligned16(Y))) || !aligned16(w->payload) || !aligned16(w->plan) ||
      (reinterpret_cast<uintptr_t>(bias) & 3u))
    return BSP_ERR_ALIGN;
  ConvParams p;
  p.X = X;
  p.Y = Y;
  p.bias = bias;
  p.payload = w->payload;
  p.plan = (const int32_t*)w->plan;
  p.row_ptr = w->row_ptr;
  p.col_idx = w->col_idx;
  p.B = B;
  p.L = L;
  p.J = J;
  p.I = w->I;
  p.O = w->O;
  p.H = w->H;
  p.K = w->K;
  p.M = (int32_t)M;
  p.N = (int32_t)N;
  p.sh = sh;
  p.sw = sw;
  p.ph = ph;
  p.pw = pw;
  p.P = (int32_t)((int64_t)B * M * N);
  p.residual = nullptr;
  p.relu = 0;
  *out = p;
  return BSP_OK;
}

}  // namespace

namespace {

// The library's own scratch memory for the partial sums of FC layers cut along their input
// channels: allocated on first need, kept, grown when a larger layer comes (one device).
float* g_fc_scratch = nullptr;
int64_t g_fc_scratch_bytes = 0;

int launch_fc_xlds(const ConvParams& p, const bsp_weights* w, hipStream_t st) {
  int64_t need = 0;
  int rc = bsp_launch_fc_xlds(p, w->dtype, w->bo, w->bi, g_fc_scratch, g_fc_scratch_bytes, &need, st);
  if (rc != BSP_ERR_CAPACITY) return rc;
  // (under stream capture this allocation fails: run the layer once before capturing it)
  if (g_fc_scratch) (void)hipFree(g_fc_scratch);
  g_fc_scratch = nullptr;
  g_fc_scratch_bytes = 0;
  if (hipMalloc((void**)&g_fc_scratch, (size_t)need) != hipSuccess) {
    (void)hipGetLastError();
    return BSP_ERR_HIP;
  }
  g_fc_scratch_bytes = need;
  return bsp_launch_fc_xlds(p, w->dtype, w->bo, w->bi, g_fc_scratch, g_fc_scratch_bytes, &need, st);
}

// Scratch memory handed in by the caller of dispatch instead of the library's own.
struct FixedScratch {
  float* ptr;
  int64_t bytes;
};

int dispatch(const bsp_weights* w, const ConvParams& p, void* stream, const FixedScratch* fixed = nullptr) {
  if (p.P == 0) return BSP_OK;
  const int allow = w->kernels ? w->kernels : ~0;
  if (w->dtype == BSP_BF16) {
    // each launcher declines (UNSUPPORTED, nothing launched) what lies outside its limits
    const bool chunked = bsp_tile_supported(p, w->dtype);  // whole 8-channel chunks
    hipStream_t st = (hipStream_t)stream;
    int rc = BSP_ERR_UNSUPPORTED;
    if (chunked && (allow & BSP_KERNEL_FC)) {
      int64_t need = 0;
      rc = fixed ? bsp_launch_fc_xlds(p, w->dtype, w->bo, w->bi, fixed->ptr, fixed->bytes, &need, st)
                 : launch_fc_xlds(p, w, st);
    }
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    if (chunked && (allow & BSP_KERNEL_FC)) rc = bsp_launch_fc_stream(p, w->dtype, w->bo, w->bi, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    // The row-band kernels take the layers they were measured to be faster on (per-shape
    // timings of the ResNet50-shaped layers): windows with at least 128 input channels, and
    // pointwise layers with 128..512 input channels, at least 128 output channels and fewer
    // than 100 000 pixels.  A caller's kernel mask overrides the rule.
    if ((allow & BSP_KERNEL_PW) && p.H == 1 && p.K == 1) rc = bsp_launch_pw(p, w->dtype, w->plan_host, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    if ((allow & BSP_KERNEL_BAND) && p.H == 3 && p.K == 3) rc = bsp_launch_band(p, w->dtype, w->plan_host, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    const bool rows_pick = p.H > 1 ? p.I >= 128
                                   : (p.I >= 128 && p.I <= 512 && p.O >= 128 && p.P < 100000);
    if ((allow & BSP_KERNEL_ROWS) && (rows_pick || w->kernels)) rc = bsp_launch_rows(p, w->dtype, w->plan_host, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    if ((allow & BSP_KERNEL_FIRST) && p.I <= 4) rc = bsp_launch_first(p, w->dtype, w->plan_host, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    if (allow & BSP_KERNEL_LDS) rc = bsp_launch_lds(p, w->dtype, w->plan_host, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
    if (chunked && (allow & BSP_KERNEL_TILE)) rc = bsp_launch_tile(p, w->dtype, st);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
  }
  return bsp_launch_general(p, w->dtype, w->bo, w->bi, (hipStream_t)stream);
}

}  // namespace

// The scratch memory of bsp_fc_fused_static: part of the library's image on every GPU it runs
// on, there until the process ends.  In host code this name only stands for the array (its
// device address comes from hipGetSymbolAddress, once per device).
constexpr int64_t kStaticScratchBytes = 4ll << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// The array's address on the current device.
int static_scratch(float** out) {
  static float* ptr[64] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return BSP_ERR_HIP;
  if (dev < 0 || dev >= 64) return BSP_ERR_UNSUPPORTED;
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return BSP_ERR_HIP;
    }
    ptr[dev] = (float*)p;
  }
  *out = ptr[dev];
  return BSP_OK;
}

}  // namespace

extern "C" {

int bsp_fc_fused_static(const bsp_weights* w, const void* X, const float* bias, const void* residual,
                        int32_t relu, void* Y, int32_t B, void* stream) {
  if (!w || (B != 0 && (!X || !Y))) return BSP_ERR_NULL;
  if (w->H != 1 || w->K != 1) return BSP_ERR_SHAPE;
  ConvParams p;
  if (int rc = prepare(w, X, bias, Y, B, 1, 1, 1, 1, 0, 0, &p)) return rc;
  if (residual && !aligned16(residual)) return BSP_ERR_ALIGN;
  p.residual = residual;
  p.relu = relu != 0;
  FixedScratch fixed{nullptr, kStaticScratchBytes};
  if (int rc = static_scratch(&fixed.ptr)) return rc;
  return dispatch(w, p, stream, &fixed);
}

int bsp_conv2d_general(const bsp_weights* w, const void* X, const float* bias, void* Y,
                       int32_t B, int32_t L, int32_t J, int32_t stride_h, int32_t stride_w,
                       int32_t pad_h, int32_t pad_w, void* stream) {
  ConvParams p;
  if (int rc = prepare(w, X, bias, Y, B, L, J, stride_h, stride_w, pad_h, pad_w, &p)) return rc;
  if (p.P == 0) return BSP_OK;
  return bsp_launch_general(p, w->dtype, w->bo, w->bi, (hipStream_t)stream);
}

int bsp_bottleneck(const bsp_weights* w1, const bsp_weights* w2, const bsp_weights* w3, const void* X,
                   const float* bias1, const float* bias2, const float* bias3, const void* residual,
                   int32_t relu, void* Y, int32_t B, int32_t L, int32_t J, void* stream) {
  if (!w1 || !w2 || !w3) return BSP_ERR_NULL;
  for (const bsp_weights* w : {w1, w2, w3}) {
    if (!w->plan || !w->plan_host) return BSP_ERR_NULL;
    if (w->dtype != BSP_BF16) return w->dtype == BSP_F32 ? BSP_ERR_UNSUPPORTED : BSP_ERR_DTYPE;
    if (!aligned16(w->plan)) return BSP_ERR_ALIGN;
  }
  if (B < 0 || L < 1 || J < 1) return BSP_ERR_SHAPE;
  if (B == 0) return BSP_OK;
  if (!X || !Y) return BSP_ERR_NULL;
  if (!aligned16(X) || !aligned16(Y) || (residual && !aligned16(residual))) return BSP_ERR_ALIGN;
  for (const float* b : {bias1, bias2, bias3})
    if (reinterpret_cast<uintptr_t>(b) & 3u) return BSP_ERR_ALIGN;
  return bsp_launch_chain(w1, w2, w3, X, bias1, bias2, bias3, residual, Y, B, L, J, relu != 0,
                          (hipStream_t)stream);
}

int bsp_conv2d_only(const bsp_weights* w, const void* X, const float* bias, const void* residual,
                    int32_t relu, void* Y, int32_t B, int32_t L, int32_t J, int32_t stride_h,
                    int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t family, void* stream) {
  ConvParams p;
  if (int rc = prepare(w, X, bias, Y, B, L, J, stride_h, stride_w, pad_h, pad_w, &p)) return rc;
  if (residual && !aligned16(residual)) return BSP_ERR_ALIGN;
  p.residual = residual;
  p.relu = relu != 0;
  if (p.P == 0) return BSP_OK;
  hipStream_t st = (hipStream_t)stream;
  if (family == 0) return bsp_launch_general(p, w->dtype, w->bo, w->bi, st);
  if (w->dtype != BSP_BF16) return BSP_ERR_UNSUPPORTED;
  const bool chunked = bsp_tile_supported(p, w->dtype);
  switch (family) {
    case BSP_KERNEL_ROWS: return bsp_launch_rows(p, w->dtype, w->plan_host, st);
    case BSP_KERNEL_PW: return bsp_launch_pw(p, w->dtype, w->plan_host, st);
    case BSP_KERNEL_BAND: return bsp_launch_band(p, w->dtype, w->plan_host, st);
    case BSP_KERNEL_LDS: return bsp_launch_lds(p, w->dtype, w->plan_host, st);
    case BSP_KERNEL_FIRST: return bsp_launch_first(p, w->dtype, w->plan_host, st);
    case BSP_KERNEL_TILE: return chunked ? bsp_launch_tile(p, w->dtype, st) : BSP_ERR_UNSUPPORTED;
    case BSP_KERNEL_FC: {
      if (!chunked) return BSP_ERR_UNSUPPORTED;
      const int rc = launch_fc_xlds(p, w, st);
      return rc != BSP_ERR_UNSUPPORTED ? rc : bsp_launch_fc_stream(p, w->dtype, w->bo, w->bi, st);
    }
    default: return BSP_ERR_UNSUPPORTED;
  }
}

int bsp_conv2d(const bsp_weights* w, const void* X, const float* bias, void* Y, int32_t B,
               int32_t L, int32_t J, int32_t stride_h, int32_t stride_w, int32_t pad_h,
               int32_t pad_w, void* stream) {
  return bsp_conv2d_fused(w, X, bias, nullptr, 0, Y, B, L, J, stride_h, stride_w, pad_h, pad_w,
                          stream);
}

int bsp_conv2d_fused(const bsp_weights* w, const void* X, const float* bias,
                     const void* residual, int32_t relu, void* Y, int32_t B, int32_t L,
                     int32_t J, int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                     void* stream) {
  ConvParams p;
  if (int rc = prepare(w, X, bias, Y, B, L, J, stride_h, stride_w, pad_h, pad_w, &p)) return rc;
  if (residual && !aligned16(residual)) return BSP_ERR_ALIGN;
  p.residual = residual;
  p.relu = relu != 0;
  return dispatch(w, p, stream);
}

int bsp_fc_fused(const bsp_weights* w, const void* X, const float* bias, const void* residual,
                 int32_t relu, void* Y, int32_t B, void* stream) {
  if (!w || (B != 0 && (!X || !Y))) return BSP_ERR_NULL;
  if (w->H != 1 || w->K != 1) return BSP_ERR_SHAPE;
  return bsp_conv2d_fused(w, X, bias, residual, relu, Y, B, 1, 1, 1, 1, 0, 0, stream);
}

int bsp_fc(const bsp_weights* w, const void* X, const float* bias, void* Y, int32_t B,
           void* stream) {
  if (!w || (B != 0 && (!X || !Y))) return BSP_ERR_NULL;
  if (w->H != 1 || w->K != 1) return BSP_ERR_SHAPE;
  return bsp_conv2d(w, X, bias, Y, B, 1, 1, 1, 1, 0, 0, stream);
}

int bsp_conv2d_i8(const bsp_weights* w, const int8_t* X, const int32_t* bias, void* Y,
                  int32_t y_dtype, int32_t shift, int32_t B, int32_t L, int32_t J,
                  int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                  void* stream) {
  ConvParams p;
  if (int rc = prepare(w, X, (const float*)bias, Y, B, L, J, stride_h, stride_w, pad_h, pad_w, &p,
                       true))
    return rc;
  if (y_dtype != BSP_I8 && y_dtype != BSP_I32) return BSP_ERR_DTYPE;
  if (y_dtype == BSP_I8 && (shift < 0 || shift > 31)) return BSP_ERR_SHAPE;
  if (p.P == 0) return BSP_OK;
  if (y_dtype == BSP_I8 && (!w->kernels || (w->kernels & BSP_KERNEL_LDS)) && aligned16(X)) {
    const int rc = bsp_launch_lds_i8(p, w->plan_host, shift, (hipStream_t)stream);
    if (rc != BSP_ERR_UNSUPPORTED) return rc;
  }
  return bsp_launch_i8(p, y_dtype == BSP_I8, y_dtype == BSP_I8 ? shift : 0, w->bo, w->bi,
                       (hipStream_t)stream);
}

int bsp_fc_i8(const bsp_weights* w, const int8_t* X, const int32_t* bias, void* Y,
              int32_t y_dtype, int32_t shift, int32_t B, void* stream) {
  if (!w || (B != 0 && (!X || !Y))) return BSP_ERR_NULL;
  if (w->H != 1 || w->K != 1) return BSP_ERR_SHAPE;
  return bsp_conv2d_i8(w, X, bias, Y, y_dtype, shift, B, 1, 1, 1, 1, 0, 0, stream);
}

}  // extern "C"
