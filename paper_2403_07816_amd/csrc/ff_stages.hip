// Dispatch of the expert-FFN stages to the kernels that implement them:
// fp32 -> plain FMA path, bf16 -> MFMA path.
#include "common.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"

namespace btx {

size_t ff_scratch_bytes(int dtype, int R, int f) {
  return align_up((size_t)R * f * sizeof(float), 256);  // dys W2^T before its elementwise step
}

// The MFMA kernels need d and f to be multiples of 32; other bf16 shapes take the plain path.
static bool mfma_shape(int d, int f) { return d % 32 == 0 && f % 32 == 0 && d >= 64 && f >= 64; }

int ff_prepare() { return mfma_prepare(); }

bool ff_rows_supported(int dtype, int R, int d, int f, int E) {
  if (dtype == BTX_BF16 && mfma_shape(d, f)) return mfma_rows_ok(R, E);
  return generic_rows_ok(R, E);
}

bool ff_dw_transposed(int dtype, int d, int f) { return dtype == BTX_BF16 && mfma_shape(d, f); }
int ff_dw_pitch(int R, int E) { return mfma_dw_pitch(R, E); }

bool ff_gather_fused(int dtype, int T, int d, int f) {
  return dtype == BTX_BF16 && mfma_shape(d, f) && mfma_gather_ok(T, d);
}

bool ff_up_needs_h(int dtype, int d, int f) { return !(dtype == BTX_BF16 && mfma_shape(d, f)); }

int bwd_act_partials(int dtype, int d, int f) { return dtype == BTX_BF16 && mfma_shape(d, f) ? mfma_bwd_act_partials(f) : 1; }

int launch_up_swiglu(int dtype, const RowSource& xs, const void* W1, const void* W3, const int32_t* offsets,
                     const FfShapes& sh, void* h1, void* h3, void* act, void* partial, hipStream_t s) {
  if (dtype == BTX_BF16 && mfma_shape(sh.d, sh.f)) return mfma_up_swiglu(xs, W1, W3, offsets, sh, h1, h3, act, partial, s);
  if (xs.perm) return BTX_ERR_UNSUPPORTED;  // the plain path takes gathered rows
  return generic_up_swiglu(dtype, xs.base, W1, W3, offsets, sh, h1, h3, act, s);
}
size_t ff_split_bytes(int dtype, int d, int f) { return dtype == BTX_BF16 && mfma_shape(d, f) ? mfma_split_bytes() : 0; }

int launch_down(int dtype, const void* act, const void* W2, const int32_t* offsets, const FfShapes& sh, void* y,
                void* partial, hipStream_t s) {
  if (dtype == BTX_BF16 && mfma_shape(sh.d, sh.f)) return mfma_down(act, W2, offsets, sh, y, partial, s);
  return generic_down(dtype, act, W2, offsets, sh, y, s);
}
int launch_bwd_act(int dtype, const RowSource& dys, const void* W2, const void* h1, const void* h3, const float* gates,
                   const int32_t* perm, const int32_t* offsets, const FfShapes& sh, void* dh1, void* dh3, void* ga,
                   bool want_dw, float* dg_part, void* scratch, hipStream_t s) {
  if (dtype == BTX_BF16 && mfma_shape(sh.d, sh.f)) {
    return mfma_bwd_act(dys, W2, h1, h3, gates, perm, offsets, sh, dh1, dh3, want_dw ? ga : nullptr, dg_part, s);
  }
  if (dys.perm) return BTX_ERR_UNSUPPORTED;
  return generic_bwd_act(dtype, dys.base, W2, h1, h3, gates, perm, offsets, sh, dh1, dh3, ga, dg_part, scratch, s);
}
int launch_bwd_dx(int dtype, const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* offsets,
                  const FfShapes& sh, void* dxs, void* partial, hipStream_t s) {
  if (dtype == BTX_BF16 && mfma_shape(sh.d, sh.f)) return mfma_bwd_dx(dh1, dh3, W1, W3, offsets, sh, dxs, partial, s);
  return generic_bwd_dx(dtype, dh1, dh3, W1, W3, offsets, sh, dxs, s);
}
int launch_bwd_dw13(int dtype, int dW_dtype, const void* xs, const void* dh1, const void* dh3, const int32_t* offsets,
                    const FfShapes& sh, void* dW1, void* dW3, hipStream_t s) {
  if (dtype == BTX_BF16 && mfma_shape(sh.d, sh.f)) return mfma_bwd_dw13(dW_dtype, xs, dh1, dh3, offsets, sh, dW1, dW3, s);
  return generic_bwd_dw13(dtype, dW_dtype, xs, dh1, dh3, offsets, sh, dW1, dW3, s);
}
int launch_bwd_dw2(int dtype, int dW_dtype, const void* ga, const void* dys, const int32_t* offsets, const FfShapes& sh,
                   void* dW2, hipStream_t s) {
  if (dtype == BTX_BF16 && mfma_shape(sh.d, sh.f)) return mfma_bwd_dw2(dW_dtype, ga, dys, offsets, sh, dW2, s);
  return generic_bwd_dw2(dtype, dW_dtype, ga, dys, offsets, sh, dW2, s);
}

}  // namespace btx
