// Row-wise kernels: LayerNorm forward / backward, column sums for bias gradients,
// fixed-order partial reductions, copy and zero fill.  All are HBM-bound: one
// wave per row with 16-byte accesses, fp32 arithmetic, and every cross-row sum is
// taken in a fixed order (per-block partial sums, then an ascending sum over
// blocks) so that results do not depend on timing.
#include "device_common.h"
#include "kernels.h"

namespace dapple {

template <typename T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; };
template <> struct Vec<bf16> { static constexpr int N = 8; };

template <typename T>
__device__ __forceinline__ void load_vec(const T* p, float (&o)[Vec<T>::N]);
template <>
__device__ __forceinline__ void load_vec<float>(const float* p, float (&o)[4]) {
  float4 v = *(const float4*)p;
  o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
template <>
__device__ __forceinline__ void load_vec<bf16>(const bf16* p, float (&o)[8]) {
  bf16x8 v = *(const bf16x8*)p;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (float)v[e];
}
template <typename T>
__device__ __forceinline__ void store_vec(T* p, const float (&o)[Vec<T>::N]);
template <>
__device__ __forceinline__ void store_vec<float>(float* p, const float (&o)[4]) {
  *(float4*)p = make_float4(o[0], o[1], o[2], o[3]);
}
template <>
__device__ __forceinline__ void store_vec<bf16>(bf16* p, const float (&o)[8]) {
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (bf16)o[e];
  *(bf16x8*)p = v;
}

// V consecutive elements of a tensor that is either of the io type T or fp32 (the pre-LayerNorm
// sums of a bf16 stage are kept in fp32: the residual stream is never rounded to bf16)
template <typename T, bool Z32>
__device__ __forceinline__ void load_z(const void* base, long off, float (&o)[Vec<T>::N]) {
  if (Z32) {
#pragma unroll
    for (int e = 0; e < Vec<T>::N; e += 4) {
      float4 v = *(const float4*)((const float*)base + off + e);
      o[e] = v.x; o[e + 1] = v.y; o[e + 2] = v.z; o[e + 3] = v.w;
    }
  } else {
    load_vec<T>((const T*)base + off, o);
  }
}

// ------------------------------------------------------------------ LayerNorm forward
// one wave per row; NCH = ceil(H / (64 * VEC)) register chunks per lane
template <typename T, int NCH, bool Z32>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const void* __restrict__ z, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ y,
                                                     float* __restrict__ y32, float* __restrict__ stats, int rows,
                                                     int H, float eps) {
  constexpr int V = Vec<T>::N;
  int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float x[NCH][V];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    int col = (c * 64 + lane) * V;
    if (col < H) {
      load_z<T, Z32>(z, (long)row * H + col, x[c]);
#pragma unroll
      for (int e = 0; e < V; ++e) s += x[c][e];
    }
  }
  float mean = wave_sum(s) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    int col = (c * 64 + lane) * V;
    if (col < H) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        float d = x[c][e] - mean;
        q += d * d;
      }
    }
  }
  float rstd = rsqrtf(wave_sum(q) / (float)H + eps);
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    int col = (c * 64 + lane) * V;
    if (col < H) {
      float g[V], b[V], o[V];
      load_vec<T>(gamma + col, g);
      load_vec<T>(beta + col, b);
#pragma unroll
      for (int e = 0; e < V; ++e) o[e] = (x[c][e] - mean) * rstd * g[e] + b[e];
      store_vec<T>(y + (long)row * H + col, o);
      if (y32) {  // unrounded copy for the residual branch
#pragma unroll
        for (int e = 0; e < V; e += 4)
          *(float4*)(y32 + (long)row * H + col + e) = make_float4(o[e], o[e + 1], o[e + 2], o[e + 3]);
      }
    }
  }
}

// ------------------------------------------------------------------ LayerNorm backward
// A block takes LNB_ROWS consecutive rows (each wave every 4th of them), keeps the
// per-column partial sums of dy*xhat, dy and dz in registers, combines the four
// waves in LDS in wave order and writes partial[(blk*3 + v)*H + col].
constexpr int LNB_ROWS = 8;

template <typename T, int NCH, bool Z32>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T* __restrict__ dy, const void* __restrict__ z,
                                                     const float* __restrict__ stats, const T* __restrict__ gamma,
                                                     T* __restrict__ dz, float* __restrict__ partial, int rows, int H) {
  constexpr int V = Vec<T>::N;
  extern __shared__ __attribute__((aligned(16))) float red[];  // [4 waves][3][H]
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float pg[NCH][V], pb[NCH][V], pz[NCH][V], g[NCH][V];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    int col = (c * 64 + lane) * V;
#pragma unroll
    for (int e = 0; e < V; ++e) pg[c][e] = pb[c][e] = pz[c][e] = g[c][e] = 0.f;
    if (col < H) load_vec<T>(gamma + col, g[c]);
  }
  // each wave takes rows wave, wave + 4, ...; the loads of all its rows are issued first
  constexpr int RPW = LNB_ROWS / 4;
  float d[RPW][NCH][V], zz[RPW][NCH][V], mean[RPW], rstd[RPW];
  bool live[RPW];
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    int row = blockIdx.x * LNB_ROWS + wave + 4 * q;
    live[q] = row < rows;
    mean[q] = live[q] ? stats[2 * row] : 0.f;
    rstd[q] = live[q] ? stats[2 * row + 1] : 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      int col = (c * 64 + lane) * V;
      if (live[q] && col < H) {
        load_vec<T>(dy + (long)row * H + col, d[q][c]);
        load_z<T, Z32>(z, (long)row * H + col, zz[q][c]);
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) d[q][c][e] = zz[q][c][e] = 0.f;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    if (!live[q]) continue;
    int row = blockIdx.x * LNB_ROWS + wave + 4 * q;
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      int col = (c * 64 + lane) * V;
      if (col < H) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          zz[q][c][e] = (zz[q][c][e] - mean[q]) * rstd[q];  // x-hat
          float dxh = d[q][c][e] * g[c][e];
          s1 += dxh;
          s2 += dxh * zz[q][c][e];
        }
      }
    }
    float m1 = wave_sum(s1) / (float)H, m2 = wave_sum(s2) / (float)H;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      int col = (c * 64 + lane) * V;
      if (col < H) {
        float o[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
          o[e] = rstd[q] * (d[q][c][e] * g[c][e] - m1 - zz[q][c][e] * m2);
          pg[c][e] += d[q][c][e] * zz[q][c][e];
          pb[c][e] += d[q][c][e];
        }
        store_vec<T>(dz + (long)row * H + col, o);
        // the bias gradient of the producing linear sums dz as it is stored
#pragma unroll
        for (int e = 0; e < V; ++e) pz[c][e] += to_f32(from_f32<T>(o[e]));
      }
    }
  }
  // combine the four waves in wave order, ((w0 + w1) + w2) + w3, with 16-byte LDS accesses
  float* mine = red + wave * 3 * H;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    int col = (c * 64 + lane) * V;
    if (col < H) {
#pragma unroll
      for (int e = 0; e < V; e += 4) {
        *(float4*)(mine + 0 * H + col + e) = make_float4(pg[c][e], pg[c][e + 1], pg[c][e + 2], pg[c][e + 3]);
        *(float4*)(mine + 1 * H + col + e) = make_float4(pb[c][e], pb[c][e + 1], pb[c][e + 2], pb[c][e + 3]);
        *(float4*)(mine + 2 * H + col + e) = make_float4(pz[c][e], pz[c][e + 1], pz[c][e + 2], pz[c][e + 3]);
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x * 4; i < 3 * H; i += 256 * 4) {
    float4 a = *(const float4*)(red + i), b = *(const float4*)(red + 3 * H + i);
    float4 c2 = *(const float4*)(red + 6 * H + i), d2 = *(const float4*)(red + 9 * H + i);
    float4 r;
    r.x = ((a.x + b.x) + c2.x) + d2.x;
    r.y = ((a.y + b.y) + c2.y) + d2.y;
    r.z = ((a.z + b.z) + c2.z) + d2.z;
    r.w = ((a.w + b.w) + c2.w) + d2.w;
    *(float4*)(partial + (long)blockIdx.x * 3 * H + i) = r;
  }
}

// out_v[c] += sum over blocks of partial[(blk*nvec + v)*H + c].  A workgroup takes 64
// columns; wave w adds blocks w, w+4, w+8, ... in ascending order and the four wave sums
// are combined as ((s0 + s1) + s2) + s3: a fixed order, independent of timing.
__global__ __launch_bounds__(256) void partial_reduce_kernel(const float* __restrict__ partial, int nblk, int nvec,
                                                             int H, float* o0, float* o1, float* o2, long zs_partial,
                                                             long zs_out, int PS) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const int v = blockIdx.y;
  float* o = v == 0 ? o0 : (v == 1 ? o1 : o2);
  if (!o) return;
  o += blockIdx.z * zs_out;
  partial += blockIdx.z * zs_partial;
  float t = 0.f;
  if (c < H) {
    const float* p = partial + (long)v * PS + c;  // PS: row stride of the partial blocks
    const long stride = (long)nvec * PS;
    int b = w;
    for (; b + 28 < nblk; b += 32) {
      float x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) x[u] = p[(long)(b + 4 * u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) t += x[u];
    }
    for (; b < nblk; b += 4) t += p[(long)b * stride];
  }
  red[w][lane] = t;
  __syncthreads();
  if (w == 0 && c < H) {
    float r = red[0][lane] + red[1][lane];
    r += red[2][lane];
    r += red[3][lane];
    o[c] += r;
  }
}

// Several partial_reduce jobs in one launch (blockIdx.y = job): the summation of a job is that of
// partial_reduce_kernel, addition for addition.
__global__ __launch_bounds__(256) void reduce_jobs_kernel(ReduceJobs J) {
  __shared__ float red[4][64];
  const ReduceJob& job = J.j[blockIdx.y];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  if (blockIdx.x * 64 >= job.cols) return;   // the whole workgroup: no barrier is skipped by part of it
  float t = 0.f;
  if (c < job.cols) {
    const float* p = job.partial + c;
    const long stride = job.stride;
    const int nblk = job.nblk;
    int b = w;
    for (; b + 28 < nblk; b += 32) {
      float x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) x[u] = p[(long)(b + 4 * u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) t += x[u];
    }
    for (; b < nblk; b += 4) t += p[(long)b * stride];
  }
  red[w][lane] = t;
  __syncthreads();
  if (w == 0 && c < job.cols) {
    float r = red[0][lane] + red[1][lane];
    r += red[2][lane];
    r += red[3][lane];
    job.out[c] += r;
  }
}

// ------------------------------------------------------------------ column sums
constexpr int CS_ROWS = 64;
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ X, int rows, int cols, int ld,
                                                     float* __restrict__ partial, long zs_x, int PS) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4][64 * V];
  X += blockIdx.z * zs_x;
  partial += (long)blockIdx.z * gridDim.y * PS;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int col = (blockIdx.x * 64 + lane) * V;
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  if (col < cols) {
    // all of the wave's loads are issued before the first add (rows past the end re-read the
    // last row and are masked), so the kernel is bound by bandwidth instead of by 16 round trips
    const int r0 = blockIdx.y * CS_ROWS;
    constexpr int RPW = CS_ROWS / 4;
    float x[RPW][V];
#pragma unroll
    for (int q = 0; q < RPW; ++q) {
      int row = r0 + wave + 4 * q;
      load_vec<T>(X + (long)(row < rows ? row : rows - 1) * ld + col, x[q]);
    }
#pragma unroll
    for (int q = 0; q < RPW; ++q) {
      const float m = (r0 + wave + 4 * q) < rows ? 1.f : 0.f;
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += m * x[q][e];
    }
  }
#pragma unroll
  for (int e = 0; e < V; ++e) red[wave][lane * V + e] = acc[e];
  __syncthreads();
  if (wave == 0 && col < cols) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      float t = red[0][lane * V + e] + red[1][lane * V + e];
      t += red[2][lane * V + e];
      t += red[3][lane * V + e];
      partial[(long)blockIdx.y * PS + col + e] = t;
    }
  }
}

__global__ void zero_kernel(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}
__global__ void copy_kernel(uint4* d, const uint4* s, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) d[i] = s[i];
}

// ------------------------------------------------------------------ launchers
template <typename T>
static int nch_for(int H) {
  int per = 64 * Vec<T>::N;
  return (H + per - 1) / per;
}

template <typename T, bool Z32>
static hipError_t ln_fwd_t(const void* z, const void* g, const void* b, void* y, float* y32, float* stats, int rows,
                           int H, float eps, hipStream_t st) {
  dim3 grid((rows + 3) / 4), blk(256);
  int n = nch_for<T>(H);
#define LNF(N)                                                                                                \
  hipLaunchKernelGGL((ln_fwd_kernel<T, N, Z32>), grid, blk, 0, st, z, (const T*)g, (const T*)b, (T*)y, y32, stats, \
                     rows, H, eps)
  if (n <= 1) LNF(1);
  else if (n <= 2) LNF(2);
  else if (n <= 4) LNF(4);
  else if (n <= 8) LNF(8);
  else return hipErrorInvalidValue;
#undef LNF
  return hipGetLastError();
}

hipError_t launch_ln_fwd(Dtype dt, const void* z, bool z_f32, const void* gamma, const void* beta, void* y,
                         float* y32, float* stats, int rows, int H, float eps, hipStream_t st) {
  if (dt != DT_BF16) return ln_fwd_t<float, false>(z, gamma, beta, y, y32, stats, rows, H, eps, st);
  return z_f32 ? ln_fwd_t<bf16, true>(z, gamma, beta, y, y32, stats, rows, H, eps, st)
               : ln_fwd_t<bf16, false>(z, gamma, beta, y, y32, stats, rows, H, eps, st);
}

template <typename T, int N, bool Z32>
static hipError_t ln_bwd_launch(const void* dy, const void* z, const float* stats, const void* g, void* dz,
                                float* partial, int nb, int rows, int H, hipStream_t st) {
  // up to 96 KiB of LDS for the widest rows; set once per instantiation by whichever host thread comes first
  // (initialisation of a function-local static is thread-safe)
  static const hipError_t attr_rc = hipFuncSetAttribute((const void*)ln_bwd_kernel<T, N, Z32>,
                                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                                        12 * 64 * Vec<T>::N * N * 4);
  if (attr_rc != hipSuccess) return attr_rc;
  size_t sh = (size_t)12 * H * sizeof(float);
  hipLaunchKernelGGL((ln_bwd_kernel<T, N, Z32>), dim3(nb), dim3(256), sh, st, (const T*)dy, z, stats, (const T*)g,
                     (T*)dz, partial, rows, H);
  return hipGetLastError();
}

template <typename T, bool Z32>
static hipError_t ln_bwd_t(const void* dy, const void* z, const float* stats, const void* g, void* dz,
                           float* partial, int nb, int rows, int H, hipStream_t st) {
  int n = nch_for<T>(H);
  if (n <= 1) return ln_bwd_launch<T, 1, Z32>(dy, z, stats, g, dz, partial, nb, rows, H, st);
  if (n <= 2) return ln_bwd_launch<T, 2, Z32>(dy, z, stats, g, dz, partial, nb, rows, H, st);
  if (n <= 4) return ln_bwd_launch<T, 4, Z32>(dy, z, stats, g, dz, partial, nb, rows, H, st);
  return hipErrorInvalidValue;
}

hipError_t launch_ln_bwd(Dtype dt, const void* dy, const void* z, bool z_f32, const float* stats, const void* gamma,
                         void* dz, float* partial, int* nblk, int rows, int H, hipStream_t st) {
  int nb = (rows + LNB_ROWS - 1) / LNB_ROWS;
  *nblk = nb;
  if (dt != DT_BF16) return ln_bwd_t<float, false>(dy, z, stats, gamma, dz, partial, nb, rows, H, st);
  return z_f32 ? ln_bwd_t<bf16, true>(dy, z, stats, gamma, dz, partial, nb, rows, H, st)
               : ln_bwd_t<bf16, false>(dy, z, stats, gamma, dz, partial, nb, rows, H, st);
}

hipError_t launch_partial_reduce(const float* partial, int nblk, int nvec, int H, float* o0, float* o1, float* o2,
                                 hipStream_t st) {
  dim3 grid((H + 63) / 64, nvec), blk(256);
  hipLaunchKernelGGL(partial_reduce_kernel, grid, blk, 0, st, partial, nblk, nvec, H, o0, o1, o2, 0L, 0L, H);
  return hipGetLastError();
}

hipError_t launch_colsum(Dtype dt, const void* X, int rows, int cols, int ld, float* partial, float* out, int nb,
                         long zs_x, long zs_out, hipStream_t st) {
  int nrb = (rows + CS_ROWS - 1) / CS_ROWS;
  int vec = dt == DT_BF16 ? 8 : 4;
  int PS = (cols + vec - 1) / vec * vec;  // whole vectors: the last one may reach into X's row padding (ld >= PS)
  if (dt == DT_BF16) {
    dim3 grid((cols + 64 * 8 - 1) / (64 * 8), nrb, nb);
    hipLaunchKernelGGL(colsum_kernel<bf16>, grid, dim3(256), 0, st, (const bf16*)X, rows, cols, ld, partial, zs_x, PS);
  } else {
    dim3 grid((cols + 64 * 4 - 1) / (64 * 4), nrb, nb);
    hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)X, rows, cols, ld, partial, zs_x, PS);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid((cols + 63) / 64, 1, nb);
  hipLaunchKernelGGL(partial_reduce_kernel, grid, dim3(256), 0, st, partial, nrb, 1, cols, out, nullptr, nullptr,
                     (long)nrb * PS, zs_out, PS);
  return hipGetLastError();
}

hipError_t launch_colsum_partials(Dtype dt, const void* X, int rows, int cols, int ld, float* partial, int nb, long zs_x,
                                  int* nblk, int* PS_out, hipStream_t st) {
  int nrb = (rows + CS_ROWS - 1) / CS_ROWS;
  int vec = dt == DT_BF16 ? 8 : 4;
  int PS = (cols + vec - 1) / vec * vec;
  *nblk = nrb;
  *PS_out = PS;
  if (dt == DT_BF16) {
    dim3 grid((cols + 64 * 8 - 1) / (64 * 8), nrb, nb);
    hipLaunchKernelGGL(colsum_kernel<bf16>, grid, dim3(256), 0, st, (const bf16*)X, rows, cols, ld, partial, zs_x, PS);
  } else {
    dim3 grid((cols + 64 * 4 - 1) / (64 * 4), nrb, nb);
    hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)X, rows, cols, ld, partial, zs_x, PS);
  }
  return hipGetLastError();
}

hipError_t launch_reduce_jobs(const ReduceJobs& J, hipStream_t st) {
  if (J.n <= 0) return hipSuccess;
  int maxc = 0;
  for (int i = 0; i < J.n; ++i) maxc = J.j[i].cols > maxc ? J.j[i].cols : maxc;
  dim3 grid((maxc + 63) / 64, J.n);
  hipLaunchKernelGGL(reduce_jobs_kernel, grid, dim3(256), 0, st, J);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
  size_t n16 = bytes / 16;
  if (!n16) return hipSuccess;
  int blocks = (int)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, st, (uint4*)dst, (const uint4*)src, n16);
  return hipGetLastError();
}

hipError_t launch_zero(void* dst, size_t bytes, hipStream_t st) {
  size_t n16 = bytes / 16;
  if (!n16) return hipSuccess;
  int blocks = (int)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
  hipLaunchKernelGGL(zero_kernel, dim3(blocks), dim3(256), 0, st, (uint4*)dst, n16);
  return hipGetLastError();
}

}  // namespace dapple
