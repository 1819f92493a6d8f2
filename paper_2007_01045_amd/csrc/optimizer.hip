// The Apply step of synchronous training: one Adam update of the stage's parameters from the
// gradients accumulated over the iteration's micro-batches.  One HBM-bound pass: per parameter
// it reads the gradient and the fp32 master weight and moments (16 bytes) and writes the three
// back plus the weight in the stage's dtype (and, optionally, the zeroed accumulator).
#include "device_common.h"
#include "kernels.h"

namespace dapple {

template <typename T>
__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ G, float* __restrict__ w32, float* __restrict__ m,
                                                   float* __restrict__ v, T* __restrict__ w, size_t n4, size_t n,
                                                   float lr, float beta1, float beta2, float eps, float c1, float c2,
                                                   float grad_scale, int zero_grads) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  auto upd = [&](float g, float& wv, float& mv, float& vv) {
    g *= grad_scale;
    mv = beta1 * mv + (1.f - beta1) * g;
    vv = beta2 * vv + (1.f - beta2) * g * g;
    // c1 = 1 / (1 - beta1^step), c2 = 1 / (1 - beta2^step)
    wv -= lr * (mv * c1) / (sqrtf(vv * c2) + eps);
  };
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    float4 g = ((const float4*)G)[i], wv = ((const float4*)w32)[i], mv = ((const float4*)m)[i], vv = ((const float4*)v)[i];
    upd(g.x, wv.x, mv.x, vv.x);
    upd(g.y, wv.y, mv.y, vv.y);
    upd(g.z, wv.z, mv.z, vv.z);
    upd(g.w, wv.w, mv.w, vv.w);
    ((float4*)w32)[i] = wv;
    ((float4*)m)[i] = mv;
    ((float4*)v)[i] = vv;
    // the four weights of the stage's dtype leave in one store (w is 16-byte aligned like the fp32 vectors)
    typedef T T4 __attribute__((ext_vector_type(4)));
    T4 o;
    o[0] = from_f32<T>(wv.x); o[1] = from_f32<T>(wv.y); o[2] = from_f32<T>(wv.z); o[3] = from_f32<T>(wv.w);
    *(T4*)(w + 4 * i) = o;
    if (zero_grads) ((float4*)G)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // the last n % 4 parameters
  for (size_t i = 4 * n4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    float wv = w32[i], mv = m[i], vv = v[i];
    upd(G[i], wv, mv, vv);
    w32[i] = wv; m[i] = mv; v[i] = vv;
    w[i] = from_f32<T>(wv);
    if (zero_grads) G[i] = 0.f;
  }
}

hipError_t launch_adam(Dtype dt, float* G, float* w32, float* m, float* v, void* w, size_t n, float lr, float beta1,
                       float beta2, float eps, float c1, float c2, float grad_scale, int zero_grads, hipStream_t st) {
  if (!n) return hipSuccess;
  const size_t n4 = n / 4;
  size_t blocks = (n4 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  if (dt == DT_BF16)
    hipLaunchKernelGGL(adam_kernel<bf16>, dim3((unsigned)blocks), dim3(256), 0, st, G, w32, m, v, (bf16*)w, n4, n, lr,
                       beta1, beta2, eps, c1, c2, grad_scale, zero_grads);
  else
    hipLaunchKernelGGL(adam_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, G, w32, m, v, (float*)w, n4, n, lr,
                       beta1, beta2, eps, c1, c2, grad_scale, zero_grads);
  return hipGetLastError();
}

}  // namespace dapple
