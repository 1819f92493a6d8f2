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
  // Streaming data, touched once per call: non-temporal loads and stores keep it from displacing what the
  // caches hold; a lane that has more than one vector to do (grids beyond the cap) takes four per turn,
  // sixteen 16-byte loads in flight before the first store.
  typedef float f4 __attribute__((ext_vector_type(4)));
  typedef T T4 __attribute__((ext_vector_type(4)));
  auto ld = [](const float* p, size_t i) { return __builtin_nontemporal_load((const f4*)p + i); };
  auto st = [](float* p, size_t i, f4 x) { __builtin_nontemporal_store(x, (f4*)p + i); };
  auto one = [&](size_t i, f4 g, f4 wv, f4 mv, f4 vv) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float we = wv[e], me = mv[e], ve = vv[e];
      upd(g[e], we, me, ve);
      wv[e] = we; mv[e] = me; vv[e] = ve;
    }
    st(w32, i, wv);
    st(m, i, mv);
    st(v, i, vv);
    // the four weights of the stage's dtype leave in one store (w is 16-byte aligned like the fp32 vectors)
    T4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = from_f32<T>(wv[e]);
    __builtin_nontemporal_store(o, (T4*)w + i);
    if (zero_grads) st(G, i, f4{0.f, 0.f, 0.f, 0.f});
  };
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n4; i += 4 * stride) {
    f4 g[4], w4[4], m4[4], v4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      g[u] = ld(G, i + u * stride); w4[u] = ld(w32, i + u * stride); m4[u] = ld(m, i + u * stride); v4[u] = ld(v, i + u * stride);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) one(i + u * stride, g[u], w4[u], m4[u], v4[u]);
  }
  for (; i < n4; i += stride) one(i, ld(G, i), ld(w32, i), ld(m, i), ld(v, i));
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
  // one vector per lane where the grid allows it: measured 5.8 TB/s against 4.9 with 8192 workgroups striding
  if (blocks > (1u << 20)) blocks = 1u << 20;
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
