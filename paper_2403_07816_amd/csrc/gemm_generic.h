// Entry points of the plain FMA grouped-GEMM path (see gemm_generic.hip).
#pragma once
#include "common.h"

namespace btx {
// the row tiles of the row-grouped products are the y dimension of the launch grid (at most 65535)
bool generic_rows_ok(int R, int E);
int generic_up_swiglu(int dtype, const void* xs, const void* W1, const void* W3, const int32_t* off, const FfShapes& sh,
                      void* h1, void* h3, void* act, hipStream_t s);
int generic_down(int dtype, const void* act, const void* W2, const int32_t* off, const FfShapes& sh, void* y,
                 hipStream_t s);
int generic_bwd_act(int dtype, const void* dys, const void* W2, const void* h1, const void* h3, const float* gates,
                    const int32_t* perm, const int32_t* off, const FfShapes& sh, void* dh1, void* dh3, void* ga,
                    float* dg_part, void* scratch, hipStream_t s);
int generic_bwd_dx(int dtype, const void* dh1, const void* dh3, const void* W1, const void* W3, const int32_t* off,
                   const FfShapes& sh, void* dxs, hipStream_t s);
int generic_bwd_dw13(int dtype, int dW_dtype, const void* xs, const void* dh1, const void* dh3, const int32_t* off,
                     const FfShapes& sh, void* dW1, void* dW3, hipStream_t s);
int generic_bwd_dw2(int dtype, int dW_dtype, const void* ga, const void* dys, const int32_t* off, const FfShapes& sh,
                    void* dW2, hipStream_t s);
}  // namespace btx
