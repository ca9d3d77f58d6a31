// AdamW step on the adapter parameters (the optimiser of the paper's hyper-parameter table;
// decoupled weight decay as in Loshchilov & Hutter).  Master parameters and both moments are
// float32; an optional copy in the storage dtype is refreshed in the same pass, so the block's
// next forward reads bf16 banks without a separate cast.
#include "common.h"

namespace mixlora {

template <typename E>
__global__ __launch_bounds__(256) void adamw_kernel(int64_t n, float *__restrict__ p,
                                                    const float *__restrict__ g,
                                                    float *__restrict__ m, float *__restrict__ v,
                                                    E *__restrict__ lowp, float lr, float beta1,
                                                    float beta2, float eps, float decay,
                                                    float inv_bc1, float inv_bc2) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x) {
    const float gi = g[i];
    float pi = p[i] * decay;                       // p <- p (1 - lr * weight_decay)
    const float mi = beta1 * m[i] + (1.f - beta1) * gi;
    const float vi = beta2 * v[i] + (1.f - beta2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    pi -= lr * (mi * inv_bc1) / (sqrtf(vi * inv_bc2) + eps);
    p[i] = pi;
    if (lowp) lowp[i] = from_f32<E>(pi);
  }
}

}  // namespace mixlora

extern "C" int mixlora_adamw_step(const mixlora_adamw *h, int64_t n, float *param,
                                  const float *grad, float *m, float *v, void *lowp,
                                  int32_t lowp_dtype, void *stream) {
  using namespace mixlora;
  if (!h || !param || !grad || !m || !v) return MIXLORA_E_NULL;
  if (lowp && lowp_dtype != MIXLORA_F32 && lowp_dtype != MIXLORA_BF16) return MIXLORA_E_DTYPE;
  if (n < 1 || h->step < 1 || !(h->beta1 >= 0.f && h->beta1 < 1.f) ||
      !(h->beta2 >= 0.f && h->beta2 < 1.f) || !(h->eps > 0.f))
    return MIXLORA_E_SHAPE;
  // bias corrections in double on the host: 1 - beta^t loses digits in float for small t
  const double bc1 = 1.0 - pow((double)h->beta1, (double)h->step);
  const double bc2 = 1.0 - pow((double)h->beta2, (double)h->step);
  const float decay = 1.f - h->lr * h->weight_decay;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (lowp && lowp_dtype == MIXLORA_BF16)
    hipLaunchKernelGGL(adamw_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, st, n, param, grad,
                       m, v, (bf16_t *)lowp, h->lr, h->beta1, h->beta2, h->eps, decay,
                       (float)(1.0 / bc1), (float)(1.0 / bc2));
  else
    hipLaunchKernelGGL(adamw_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, n, param, grad,
                       m, v, (float *)lowp, h->lr, h->beta1, h->beta2, h->eps, decay,
                       (float)(1.0 / bc1), (float)(1.0 / bc2));
  return hipGetLastError() == hipSuccess ? MIXLORA_OK : MIXLORA_E_HIP;
}
