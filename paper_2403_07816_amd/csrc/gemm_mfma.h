// Entry points of the bf16 MFMA grouped-GEMM path (see gemm_mfma.hip).
#pragma once
#include "common.h"

namespace btx {
// raises the dynamic-LDS limit of every kernel instantiation on the current device (not capturable)
int mfma_prepare();
// the weight-gradient products address 255 rows of the transposed, padded operands with 32-bit byte offsets
bool mfma_rows_ok(int R, int E);
int mfma_bwd_act_partials(int f);
// gathered A rows need every byte offset inside the source to fit 32 bits
bool mfma_gather_ok(int T, int d);
int mfma_up_swiglu(const RowSource& xs, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh,
                   void* h1, void* h3, void* act, void* partial, hipStream_t s);
// partial: mfma_split_bytes() of scratch for the K slices of the last round (NULL: tiles are never cut)
size_t mfma_split_bytes();
int mfma_down(const void* act, const void* W2, const int32_t* off, const FfShapes& sh, void* y, void* partial,
              hipStream_t s);
// dh1, dh3: [R,f]; gaT: [f][mfma_dw_pitch(R, E)], experts' rows padded with zeros to multiples of 64
// (for dW2; NULL when no weight gradients are wanted)
int mfma_bwd_act(const RowSource& dys, const void* W2, const void* h1, const void* h3, const float* gates,
                 const int32_t* perm, const int32_t* off, const FfShapes& sh, void* dh1, void* dh3, void* gaT,
                 float* dg_part, hipStream_t s);
int mfma_bwd_dx(const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* off,
                const FfShapes& sh, void* dxs, void* partial, hipStream_t s);
// xsT / dysT: [d][mfma_dw_pitch(R, E)], laid out like gaT above
int mfma_dw_pitch(int R, int E);
int mfma_bwd_dw13(int dW_dtype, const void* xsT, const void* dh1, const void* dh3, const int32_t* off,
                  const FfShapes& sh, void* dW1, void* dW3, hipStream_t s);
int mfma_bwd_dw2(int dW_dtype, const void* gaT, const void* dysT, const int32_t* off, const FfShapes& sh, void* dW2,
                 hipStream_t s);
}  // namespace btx
