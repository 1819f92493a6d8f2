// Kernels of the two optional ends of a stage.
//
// First stage (embedding block):  x = LN(E_w[id] + E_p[pos]),  pos = row % s.
//   forward : embed_gather writes e = E_w[id] + E_p[pos] (the LayerNorm kernels do the rest)
//   backward: dE_w[id] += sum of de over the rows that carry this id, added in ascending row
//             order by one wave per id (no atomics: reproducible bit for bit);
//             dE_p[pos] += sum over the sequences of the micro-batch, ascending.
//
// Last stage (masked-LM head):  the rows whose target is >= 0 are gathered (ascending) into a
//   dense block r, t = LN(GELU(r Wt + bt)), z = t E_out^T + b_out,
//   loss = loss_scale * sum_rows (logsumexp(z) - z[target]),  dz = loss_scale * (softmax(z) - onehot).
//   The products are GEMM launches; here are the compaction, the gather / scatter of rows, the
//   row-wise cross-entropy and an element-wise product.
#include "device_common.h"
#include "kernels.h"

namespace dapple {

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ void embed_gather_kernel(const int32_t* __restrict__ ids, const T* __restrict__ Ew,
                                    const T* __restrict__ Ep, T* __restrict__ e, int rows, int s, int H, int vocab) {
  int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  int id = ids[row];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);  // ids outside the table are clamped, never dereferenced
  const T* a = Ew + (long)id * H;
  const T* b = Ep + (long)(row % s) * H;
  for (int c = lane; c < H; c += 64) e[(long)row * H + c] = from_f32<T>(to_f32(a[c]) + to_f32(b[c]));
}

// one wave per row r: if r is the first row with its id, add all rows with that id in ascending order
template <typename T>
__global__ void embed_scatter_kernel(const int32_t* __restrict__ ids, const T* __restrict__ de,
                                     float* __restrict__ dEw, int rows, int H, int vocab) {
  int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  int id = ids[r];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  // an earlier row with the same id owns the sum
  for (int base = 0; base < r; base += 64) {
    int q = base + lane;
    int v = q < r ? ids[q] : -1;
    v = v < 0 ? (q < r ? 0 : -1) : (v >= vocab ? vocab - 1 : v);
    if (__ballot(q < r && v == id)) return;
  }
  for (int c0 = 0; c0 < H; c0 += 64) {
    int c = c0 + lane;
    float acc = c < H ? to_f32(de[(long)r * H + c]) : 0.f;
    for (int base = (r + 1) & ~63; base < rows; base += 64) {
      int q = base + lane;
      int v = (q > r && q < rows) ? ids[q] : -1;
      if (q > r && q < rows) v = v < 0 ? 0 : (v >= vocab ? vocab - 1 : v);
      unsigned long long m = __ballot(q > r && q < rows && v == id);
      while (m) {  // ascending rows
        int j = __builtin_ctzll(m);
        m &= m - 1;
        if (c < H) acc += to_f32(de[(long)(base + j) * H + c]);
      }
    }
    if (c < H) dEw[(long)id * H + c] += acc;
  }
}

template <typename T>
__global__ void embed_pos_grad_kernel(const T* __restrict__ de, float* __restrict__ dEp, int b, int s, int H) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)s * H) return;
  float acc = 0.f;
  for (int bi = 0; bi < b; ++bi) acc += to_f32(de[(long)bi * s * H + idx]);
  dEp[idx] += acc;
}

// ------------------------------------------------------------------ masked-LM head
// rows_idx[i], i < np: i-th row (ascending) whose target is >= 0, -1 beyond the count; tgt[i] its
// target (clamped into the vocabulary).  info[0] = count, info[1] = 1 if more than cap rows
// are predicted (the surplus is dropped and the stage reports the overflow at the next sync).
__global__ __launch_bounds__(1024) void mlm_compact_kernel(const int32_t* __restrict__ targets, int T, int cap,
                                                           int np, int vocab, int32_t* __restrict__ rows_idx,
                                                           int32_t* __restrict__ tgt, int32_t* __restrict__ info) {
  __shared__ int wave_cnt[16];
  __shared__ int running;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) running = 0;
  for (int i = tid; i < np; i += 1024) {  // all np >= cap entries, padding rows included
    rows_idx[i] = -1;
    tgt[i] = 0;
  }
  __syncthreads();
  for (int base = 0; base < T; base += 1024) {
    int r = base + tid;
    bool on = r < T && targets[r] >= 0;
    unsigned long long m = __ballot(on);
    if (lane == 0) wave_cnt[wave] = __builtin_popcountll(m);
    __syncthreads();
    int before = running;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    int pos = before + __builtin_popcountll(m & ((1ull << lane) - 1ull));
    if (on && pos < cap) {
      int t = targets[r];
      rows_idx[pos] = r;
      tgt[pos] = t >= vocab ? vocab - 1 : t;
    }
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w = 0; w < 16; ++w) tot += wave_cnt[w];
      running += tot;
    }
    __syncthreads();
  }
  if (tid == 0) {
    info[0] = running < cap ? running : cap;
    if (running > cap) info[1] = 1;
  }
}

// dst[i] = idx[i] >= 0 ? src[idx[i]] : 0   (rows of H elements)
template <typename T>
__global__ void gather_rows_kernel(const T* __restrict__ src, const int32_t* __restrict__ idx, T* __restrict__ dst,
                                   int n, int H, int nsrc) {
  int lane = threadIdx.x & 63, i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= n) return;
  int r = idx[i];
  bool ok = r >= 0 && r < nsrc;
  for (int c = lane; c < H; c += 64) dst[(long)i * H + c] = ok ? src[(long)r * H + c] : from_f32<T>(0.f);
}
// dst[idx[i]] = src[i] for idx[i] >= 0  (dst zeroed beforehand; the indices are distinct)
template <typename T>
__global__ void scatter_rows_kernel(const T* __restrict__ src, const int32_t* __restrict__ idx, T* __restrict__ dst,
                                    int n, int H, int ndst) {
  int lane = threadIdx.x & 63, i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= n) return;
  int r = idx[i];
  if (r < 0 || r >= ndst) return;
  for (int c = lane; c < H; c += 64) dst[(long)r * H + c] = src[(long)i * H + c];
}

// one workgroup per gathered row: z = logits + bias over v < V; row_loss = logsumexp(z) - z[tgt];
// dz = loss_scale * (softmax(z) - onehot), zero in the padding columns and in padding rows
template <typename T>
__global__ __launch_bounds__(256) void mlm_ce_kernel(const float* __restrict__ logits, const T* __restrict__ bias,
                                                     const int32_t* __restrict__ rows_idx,
                                                     const int32_t* __restrict__ tgt, int V, int VP, float loss_scale,
                                                     T* __restrict__ dz, float* __restrict__ row_loss) {
  __shared__ float red[4];
  const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = logits + (long)i * VP;
  T* d = dz + (long)i * VP;
  if (rows_idx[i] < 0) {
    for (int v = tid; v < VP; v += 256) d[v] = from_f32<T>(0.f);
    if (tid == 0) row_loss[i] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int v = tid; v < V; v += 256) mx = fmaxf(mx, z[v] + to_f32(bias[v]));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int v = tid; v < V; v += 256) sum += __expf(z[v] + to_f32(bias[v]) - mx);
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = ((red[0] + red[1]) + red[2]) + red[3];
  const float lse = mx + __logf(sum);
  int t = tgt[i];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const float inv = 1.0f / sum;
  for (int v = tid; v < VP; v += 256) {
    float g = 0.f;
    if (v < V) {
      g = __expf(z[v] + to_f32(bias[v]) - mx) * inv;
      if (v == t) g -= 1.0f;
      g *= loss_scale;
    }
    d[v] = from_f32<T>(g);
  }
  if (tid == 0) row_loss[i] = lse - (z[t] + to_f32(bias[t]));
}

// out[0] = scale * (row_loss[0] + row_loss[1] + ...), added in index order
__global__ void loss_sum_kernel(const float* __restrict__ row_loss, int n, float scale, float* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < n; ++i) t += row_loss[i];
    out[0] = t * scale;
  }
}

template <typename T>
__global__ void mul_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ c, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) c[i] = from_f32<T>(to_f32(a[i]) * to_f32(b[i]));
}

// ------------------------------------------------------------------ launchers
hipError_t launch_embed_gather(Dtype dt, const int32_t* ids, const void* Ew, const void* Ep, void* e, int rows, int s,
                               int H, int vocab, hipStream_t st) {
  dim3 grid((rows + 3) / 4), blk(256);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(embed_gather_kernel<bf16>, grid, blk, 0, st, ids, (const bf16*)Ew, (const bf16*)Ep, (bf16*)e,
                       rows, s, H, vocab);
  else
    hipLaunchKernelGGL(embed_gather_kernel<float>, grid, blk, 0, st, ids, (const float*)Ew, (const float*)Ep,
                       (float*)e, rows, s, H, vocab);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(Dtype dt, const int32_t* ids, const void* de, float* dEw, float* dEp, int b, int s, int H,
                            int vocab, hipStream_t st) {
  int rows = b * s;
  dim3 grid((rows + 3) / 4), blk(256);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(embed_scatter_kernel<bf16>, grid, blk, 0, st, ids, (const bf16*)de, dEw, rows, H, vocab);
  else
    hipLaunchKernelGGL(embed_scatter_kernel<float>, grid, blk, 0, st, ids, (const float*)de, dEw, rows, H, vocab);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2((unsigned)(((long)s * H + 255) / 256));
  if (dt == DT_BF16) hipLaunchKernelGGL(embed_pos_grad_kernel<bf16>, g2, blk, 0, st, (const bf16*)de, dEp, b, s, H);
  else hipLaunchKernelGGL(embed_pos_grad_kernel<float>, g2, blk, 0, st, (const float*)de, dEp, b, s, H);
  return hipGetLastError();
}

hipError_t launch_mlm_compact(const int32_t* targets, int T, int cap, int np, int vocab, int32_t* rows_idx,
                              int32_t* tgt, int32_t* info, hipStream_t st) {
  hipLaunchKernelGGL(mlm_compact_kernel, dim3(1), dim3(1024), 0, st, targets, T, cap, np, vocab, rows_idx, tgt, info);
  return hipGetLastError();
}

hipError_t launch_gather_rows(Dtype dt, const void* src, const int32_t* idx, void* dst, int n, int H, int nsrc,
                              hipStream_t st) {
  dim3 grid((n + 3) / 4), blk(256);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(gather_rows_kernel<bf16>, grid, blk, 0, st, (const bf16*)src, idx, (bf16*)dst, n, H, nsrc);
  else
    hipLaunchKernelGGL(gather_rows_kernel<float>, grid, blk, 0, st, (const float*)src, idx, (float*)dst, n, H, nsrc);
  return hipGetLastError();
}

hipError_t launch_scatter_rows(Dtype dt, const void* src, const int32_t* idx, void* dst, int n, int H, int ndst,
                               hipStream_t st) {
  dim3 grid((n + 3) / 4), blk(256);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(scatter_rows_kernel<bf16>, grid, blk, 0, st, (const bf16*)src, idx, (bf16*)dst, n, H, ndst);
  else
    hipLaunchKernelGGL(scatter_rows_kernel<float>, grid, blk, 0, st, (const float*)src, idx, (float*)dst, n, H, ndst);
  return hipGetLastError();
}

hipError_t launch_mlm_ce(Dtype dt, const float* logits, const void* bias, const int32_t* rows_idx, const int32_t* tgt,
                         int n, int V, int VP, float loss_scale, void* dz, float* row_loss, float* loss_out,
                         hipStream_t st) {
  if (dt == DT_BF16)
    hipLaunchKernelGGL(mlm_ce_kernel<bf16>, dim3(n), dim3(256), 0, st, logits, (const bf16*)bias, rows_idx, tgt, V, VP,
                       loss_scale, (bf16*)dz, row_loss);
  else
    hipLaunchKernelGGL(mlm_ce_kernel<float>, dim3(n), dim3(256), 0, st, logits, (const float*)bias, rows_idx, tgt, V,
                       VP, loss_scale, (float*)dz, row_loss);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(loss_sum_kernel, dim3(1), dim3(64), 0, st, row_loss, n, loss_scale, loss_out);
  return hipGetLastError();
}

hipError_t launch_mul(Dtype dt, const void* a, const void* b, void* c, long n, hipStream_t st) {
  dim3 grid((unsigned)((n + 255) / 256)), blk(256);
  if (dt == DT_BF16) hipLaunchKernelGGL(mul_kernel<bf16>, grid, blk, 0, st, (const bf16*)a, (const bf16*)b, (bf16*)c, n);
  else hipLaunchKernelGGL(mul_kernel<float>, grid, blk, 0, st, (const float*)a, (const float*)b, (float*)c, n);
  return hipGetLastError();
}

}  // namespace dapple
