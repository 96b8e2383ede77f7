// bf16 expert GEMMs.  (Temporary: routed through the plain FMA kernels.)
#include "gemm_mfma.h"
#include "gemm_generic.h"
namespace btx {
int mfma_bwd_act_partials(int) { return 1; }
int mfma_up_swiglu(const void* xs, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh, void* h1,
                   void* h3, void* act, hipStream_t s) { return generic_up_swiglu(BTX_BF16, xs, W1, W3, off, sh, h1, h3, act, s); }
int mfma_down(const void* act, const void* W2, const int32_t* off, const FfShapes& sh, void* y, hipStream_t s) { return generic_down(BTX_BF16, act, W2, off, sh, y, s); }
int mfma_bwd_act(const void*, const void*, const void*, const void*, const float*, const int32_t*, const int32_t*, const FfShapes&, void*, void*, void*, float*, hipStream_t) { return BTX_ERR_UNSUPPORTED; }
int mfma_bwd_dx(const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh, void* dxs, hipStream_t s) { return generic_bwd_dx(BTX_BF16, dh1, dh3, W1, W3, off, sh, dxs, s); }
int mfma_bwd_dw(int dW_dtype, const void* xs, const void* dh1, const void* dh3, const void* ga, const void* dys, const int32_t* off, const FfShapes& sh, void* dW1, void* dW3, void* dW2, hipStream_t s) { return generic_bwd_dw(BTX_BF16, dW_dtype, xs, dh1, dh3, ga, dys, off, sh, dW1, dW3, dW2, s); }
}
