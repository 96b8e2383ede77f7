// Fused AdamW update (Sec. 4.1 names the optimizer and its weight decay): one streaming pass
// over fp32 master weights, both moments and the gradient, which also writes the bf16 working
// copy the layer reads.  HBM-bound: 24 bytes read/written per element for p, m, v plus the
// gradient (2 or 4) and the working copy (2).
#include "common.h"

namespace btx {
namespace {

struct AdamArgs {
  float lr, beta1, beta2, eps, wd, c1, c2;   // c1 = 1/(1-beta1^t), c2 = 1/(1-beta2^t)
};

__device__ __forceinline__ void adam_one(float& p, float& m, float& v, float g, const AdamArgs& a) {
  m = fmaf(a.beta1, m, (1.f - a.beta1) * g);
  v = fmaf(a.beta2, v, (1.f - a.beta2) * g * g);
  const float upd = (m * a.c1) / (sqrtf(v * a.c2) + a.eps) + a.wd * p;
  p = fmaf(-a.lr, upd, p);
}

template <typename GT>
__global__ __launch_bounds__(256) void adamw_kernel(float* __restrict__ P, float* __restrict__ M, float* __restrict__ V,
                                                    const GT* __restrict__ G, bf16_t* __restrict__ lowp, int64_t n,
                                                    AdamArgs a) {
  const int64_t n4 = n / 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    f32x4 p = reinterpret_cast<const f32x4*>(P)[i], m = reinterpret_cast<const f32x4*>(M)[i],
          v = reinterpret_cast<const f32x4*>(V)[i];
    float g[4];
    if constexpr (sizeof(GT) == 2) {
      const u32x2 w = reinterpret_cast<const u32x2*>(G)[i];
      g[0] = bf16lo(w[0]); g[1] = bf16hi(w[0]); g[2] = bf16lo(w[1]); g[3] = bf16hi(w[1]);
    } else {
      const f32x4 w = reinterpret_cast<const f32x4*>(G)[i];
      g[0] = w[0]; g[1] = w[1]; g[2] = w[2]; g[3] = w[3];
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      float pe = p[x], me = m[x], ve = v[x];
      adam_one(pe, me, ve, g[x], a);
      p[x] = pe; m[x] = me; v[x] = ve;
    }
    reinterpret_cast<f32x4*>(P)[i] = p;
    reinterpret_cast<f32x4*>(M)[i] = m;
    reinterpret_cast<f32x4*>(V)[i] = v;
    if (lowp) reinterpret_cast<u32x2*>(lowp)[i] = u32x2{pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3])};
  }
  // up to 3 trailing elements
  if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
    const int64_t i = n4 * 4 + threadIdx.x;
    float p = P[i], m = M[i], v = V[i];
    adam_one(p, m, v, Elem<GT>::ld(G + i), a);
    P[i] = p; M[i] = m; V[i] = v;
    if (lowp) lowp[i] = f32_to_bf16(p);
  }
}

}  // namespace

int launch_adamw(float* P, float* M, float* V, const void* G, int grad_dtype, void* lowp, int64_t n, int step, float lr,
                 float beta1, float beta2, float eps, float wd, hipStream_t s) {
  AdamArgs a{lr, beta1, beta2, eps, wd, (float)(1.0 / (1.0 - std::pow((double)beta1, step))),
             (float)(1.0 / (1.0 - std::pow((double)beta2, step)))};
  const int64_t n4 = n / 4;
  const unsigned blocks = (unsigned)std::min<int64_t>(std::max<int64_t>((n4 + 255) / 256, 1), 256 * 32);
  if (grad_dtype == BTX_BF16)
    adamw_kernel<bf16_t><<<blocks, 256, 0, s>>>(P, M, V, static_cast<const bf16_t*>(G), static_cast<bf16_t*>(lowp), n, a);
  else
    adamw_kernel<float><<<blocks, 256, 0, s>>>(P, M, V, static_cast<const float*>(G), static_cast<bf16_t*>(lowp), n, a);
  BTX_LAUNCH_CHECK();
  return BTX_OK;
}

}  // namespace btx
