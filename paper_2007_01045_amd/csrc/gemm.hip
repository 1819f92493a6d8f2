// GEMM kernels of the stage: every linear layer's forward, data-gradient and
// weight-gradient product is C = epilogue(sum_k A(m,k) B(n,k)) with either operand
// stored k-contiguous or k-strided.
//
//  * gemm_mfma_kernel: bf16 operands, fp32 accumulation on the gfx950 matrix
//    cores (v_mfma_f32_32x32x16_bf16).  256 threads = 4 waves in a 2x2 grid over a
//    BM x BN tile, BK = 64 per step, LDS double-buffered.  k-contiguous operands
//    sit in LDS as [row][64] with an XOR swizzle of the 16-byte chunks and are
//    read with 128-bit loads; k-strided operands sit as [k][rows+16] and are read
//    with the LDS transpose read, so no transposed copy of an activation or a
//    weight is ever made in HBM.  The MFMA is issued with the B fragment as its
//    first operand: each lane then owns 4 consecutive output columns of one
//    output row, which the epilogue stages through LDS into coalesced stores.
//  * gemm_plain_kernel: one thread per output element, fp32 accumulation in k
//    order; used for fp32 stages (the tiny configuration) and for shapes the MFMA
//    kernel does not take.
#include "device_common.h"
#include "kernels.h"

namespace dapple {

// ------------------------------------------------------------------ epilogue
template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmArgs& g, long zc, long zbias, int row, int col, float t) {
  if (g.epi & EPI_BIAS) t += to_f32(((const T*)g.bias)[zbias + col]);
  if (g.epi & EPI_ADD) t += to_f32(((const T*)g.aux)[zc + (long)row * g.ldaux + col]);
  if (g.epi & EPI_MUL) t *= to_f32(((const T*)g.aux)[zc + (long)row * g.ldaux + col]);
  long o = zc + (long)row * g.ldc + col;
  if (g.epi & EPI_GELU) {
    ((T*)g.C)[o] = from_f32<T>(gelu_f(t));
    ((T*)g.C2)[o] = from_f32<T>(gelu_grad_f(t));
  } else if (g.epi & EPI_ACC32) {
    ((float*)g.C)[o] += t;
  } else {
    ((T*)g.C)[o] = from_f32<T>(t);
  }
}

// ------------------------------------------------------------------ plain kernel
template <typename T>
__global__ void gemm_plain_kernel(GemmArgs g) {
  int col = blockIdx.x * blockDim.x + threadIdx.x;
  int row = blockIdx.y * blockDim.y + threadIdx.y;
  int z = blockIdx.z;
  if (row >= g.M || col >= g.N) return;
  const T* A = (const T*)g.A + z * g.sA;
  const T* B = (const T*)g.B + z * g.sB;
  float acc = 0.f;
  int nseg = g.K / g.kseg_len;
  for (int s = 0; s < nseg; ++s) {
    const T* As = A + s * g.segA;
    const T* Bs = B + s * g.segB;
    for (int k = 0; k < g.kseg_len; ++k) {
      if (k >= g.k_valid) break;
      float a = to_f32(g.a_kstrided ? As[(long)k * g.lda + row] : As[(long)row * g.lda + k]);
      float b = to_f32(g.b_kstrided ? Bs[(long)k * g.ldb + col] : Bs[(long)col * g.ldb + k]);
      acc = fmaf(a, b, acc);
    }
  }
  epilogue_store<T>(g, z * g.sC, z * g.sBias, row, col, acc);
}

// ------------------------------------------------------------------ MFMA kernel
constexpr int BK = 64;
constexpr int TPAD = 16;  // row padding (elements) of a k-strided LDS tile

template <int R, bool KS>
struct OperandTile {
  static constexpr int NCH = R * 8 / 256;                   // 16-byte chunks per thread per k-tile
  static constexpr int LDS_ELEMS = KS ? BK * (R + TPAD) : R * BK;
  uint4 regs[NCH];

  // base: operand pointer already offset for batch and k-segment; r0: first row of the
  // tile; k0: first k inside the segment
  __device__ __forceinline__ void load(const bf16* base, int ld, int r0, int k0, int rmax, int kvalid, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int c = tid + 256 * i;
      const bf16* p;
      bool ok;
      if (!KS) {
        int row = c >> 3, kc = c & 7;
        ok = (r0 + row) < rmax;
        p = base + (long)(r0 + row) * ld + k0 + kc * 8;
      } else {
        int krow = c / (R / 8), rc = c % (R / 8);
        ok = (k0 + krow) < kvalid && (r0 + rc * 8) < rmax;
        p = base + (long)(k0 + krow) * ld + r0 + rc * 8;
      }
      regs[i] = ok ? *(const uint4*)p : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(bf16* S, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int c = tid + 256 * i;
      if (!KS) {
        int row = c >> 3, kc = c & 7;
        *(uint4*)(S + row * BK + ((kc ^ (row & 7)) << 3)) = regs[i];
      } else {
        int krow = c / (R / 8), rc = c % (R / 8);
        *(uint4*)(S + krow * (R + TPAD) + rc * 8) = regs[i];
      }
    }
  }
  // MFMA fragment for rows r0..r0+31 (lane & 31), k = kk*16 + 8*(lane>>5) + 0..7
  static __device__ __forceinline__ bf16x8 frag(const bf16* S, int r0, int kk, int lane) {
    if (!KS) {
      int row = r0 + (lane & 31);
      int kc = kk * 2 + (lane >> 5);
      return *(const bf16x8*)(S + row * BK + ((kc ^ (row & 7)) << 3));
    } else {
      int i16 = lane & 15, g16 = (lane >> 4) & 1, h = lane >> 5;
      int krow = kk * 16 + 8 * h + (i16 >> 2);
      int col = r0 + 16 * g16 + 4 * (i16 & 3);
      const bf16* p = S + krow * (R + TPAD) + col;
      return join8(lds_read_tr16(p), lds_read_tr16(p + 4 * (R + TPAD)));
    }
  }
};

template <int BM, int BN, bool AKS, bool BKS>
struct GemmTile {
  static constexpr int WM = BM / 2, WN = BN / 2, MI = WM / 32, NI = WN / 32;
  typedef OperandTile<BM, AKS> TA;
  typedef OperandTile<BN, BKS> TB;
  static constexpr int STAGE_ELEMS = TA::LDS_ELEMS + TB::LDS_ELEMS;
  static constexpr int EPI_LD = WN + 4;  // fp32 staging row
  static constexpr size_t MAIN_BYTES = 2 * (size_t)STAGE_ELEMS * sizeof(bf16);
  static constexpr size_t EPI_BYTES = 4 * (size_t)32 * EPI_LD * sizeof(float);
  static constexpr size_t LDS_BYTES = MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES;
};

template <int BM, int BN, bool AKS, bool BKS>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  typedef GemmTile<BM, BN, AKS, BKS> CFG;
  typedef typename CFG::TA TA;
  typedef typename CFG::TB TB;
  constexpr int MI = CFG::MI, NI = CFG::NI;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* lds = (bf16*)smem;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * CFG::WM, wn0 = (wave & 1) * CFG::WN;

  // tile index: consecutive workgroups land on different XCDs (round-robin over 8),
  // so give each XCD a contiguous run of tiles that share operand panels in its L2
  int bid = blockIdx.x;
  const int ntiles = tiles_m * tiles_n;
  if ((ntiles & 7) == 0) bid = (bid & 7) * (ntiles >> 3) + (bid >> 3);
  const int tm = bid / tiles_n, tn = bid % tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int z = blockIdx.z;

  const bf16* Ab = (const bf16*)g.A + z * g.sA;
  const bf16* Bb = (const bf16*)g.B + z * g.sB;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  TA ta;
  TB tb;
  const int nk = g.K / BK;
  const int tiles_per_seg = g.kseg_len / BK;

  auto issue_loads = [&](int kt) {
    int seg = kt / tiles_per_seg;
    int k0 = (kt - seg * tiles_per_seg) * BK;
    ta.load(Ab + seg * g.segA, g.lda, m0, k0, g.M, g.k_valid, tid);
    tb.load(Bb + seg * g.segB, g.ldb, n0, k0, g.N, g.k_valid, tid);
  };

  issue_loads(0);
  ta.store(lds, tid);
  tb.store(lds + TA::LDS_ELEMS, tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const bf16* As = lds + (kt & 1) * CFG::STAGE_ELEMS;
    const bf16* Bs = As + TA::LDS_ELEMS;
    if (kt + 1 < nk) issue_loads(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 a[MI], b[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = TA::frag(As, wm0 + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < NI; ++j) b[j] = TB::frag(Bs, wn0 + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      bf16* An = lds + ((kt + 1) & 1) * CFG::STAGE_ELEMS;
      ta.store(An, tid);
      tb.store(An + TA::LDS_ELEMS, tid);
    }
    __syncthreads();
  }

  // epilogue: per wave, 32 output rows at a time through an fp32 LDS staging tile.
  // acc[i][j][v]: row = wm0 + 32 i + (lane & 31), col = wn0 + 32 j + 8 (v>>2) + 4 (lane>>5) + (v&3)
  float* stg = (float*)smem + wave * 32 * CFG::EPI_LD;
  const long zc = z * g.sC, zbias = z * g.sBias;
  constexpr int C4 = CFG::WN / 4;  // float4 per staged row
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 v4 = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        *(float4*)(stg + (lane & 31) * CFG::EPI_LD + j * 32 + 8 * q + 4 * (lane >> 5)) = v4;
      }
    __syncthreads();
#pragma unroll 4
    for (int it = 0; it < 32 * C4 / 64; ++it) {
      int idx = it * 64 + lane;
      int r = idx / C4, c4 = idx % C4;
      int row = m0 + wm0 + i * 32 + r;
      int col = n0 + wn0 + c4 * 4;
      if (row < g.M && col < g.N) {
        float4 t = *(const float4*)(stg + r * CFG::EPI_LD + c4 * 4);
        if (col + 3 < g.N) {
          float tv[4] = {t.x, t.y, t.z, t.w};
          if (g.epi & EPI_BIAS) {
            bf16x4 bv = *(const bf16x4*)((const bf16*)g.bias + zbias + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) tv[e] += (float)bv[e];
          }
          if (g.epi & (EPI_ADD | EPI_MUL)) {
            bf16x4 xv = *(const bf16x4*)((const bf16*)g.aux + zc + (long)row * g.ldaux + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) tv[e] = (g.epi & EPI_ADD) ? tv[e] + (float)xv[e] : tv[e] * (float)xv[e];
          }
          long o = zc + (long)row * g.ldc + col;
          if (g.epi & EPI_GELU) {
            bf16x4 gv, gp;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              gv[e] = (bf16)gelu_f(tv[e]);
              gp[e] = (bf16)gelu_grad_f(tv[e]);
            }
            *(bf16x4*)((bf16*)g.C + o) = gv;
            *(bf16x4*)((bf16*)g.C2 + o) = gp;
          } else if (g.epi & EPI_ACC32) {
            float4* cp = (float4*)((float*)g.C + o);
            float4 c = *cp;
            c.x += tv[0]; c.y += tv[1]; c.z += tv[2]; c.w += tv[3];
            *cp = c;
          } else {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (bf16)tv[e];
            *(bf16x4*)((bf16*)g.C + o) = ov;
          }
        } else {
          float tv[4] = {t.x, t.y, t.z, t.w};
          for (int e = 0; e < 4 && col + e < g.N; ++e) epilogue_store<bf16>(g, zc, zbias, row, col + e, tv[e]);
        }
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------ host side
template <int BM, int BN, bool AKS, bool BKS>
static hipError_t launch_mfma(const GemmArgs& g, hipStream_t st) {
  typedef GemmTile<BM, BN, AKS, BKS> CFG;
  static bool attr_set = false;
  auto kern = gemm_mfma_kernel<BM, BN, AKS, BKS>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)CFG::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  dim3 grid(tiles_m * tiles_n, 1, g.batch);
  hipLaunchKernelGGL(kern, grid, dim3(256), CFG::LDS_BYTES, st, g, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN>
static hipError_t launch_mfma_layout(const GemmArgs& g, hipStream_t st) {
  if (g.a_kstrided) {
    return g.b_kstrided ? launch_mfma<BM, BN, true, true>(g, st) : launch_mfma<BM, BN, true, false>(g, st);
  }
  return g.b_kstrided ? launch_mfma<BM, BN, false, true>(g, st) : launch_mfma<BM, BN, false, false>(g, st);
}

static bool aligned_to(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

bool gemm_uses_mfma(Dtype dt, const GemmArgs& g) {
  if (dt != DT_BF16) return false;
  if (g.K < BK || g.K % BK || g.kseg_len % BK || g.K % g.kseg_len) return false;
  if (g.lda % 8 || g.ldb % 8 || g.ldc % 4) return false;
  if (g.sA % 8 || g.sB % 8 || g.sC % 4 || g.sBias % 4 || g.segA % 8 || g.segB % 8) return false;
  if (!aligned_to(g.A, 16) || !aligned_to(g.B, 16) || !aligned_to(g.C, 16)) return false;
  if (g.a_kstrided && g.M % 8) return false;
  if (g.b_kstrided && g.N % 8) return false;
  if ((g.epi & (EPI_ADD | EPI_MUL)) && (g.ldaux % 4 || !aligned_to(g.aux, 8))) return false;
  if ((g.epi & EPI_BIAS) && !aligned_to(g.bias, 8)) return false;
  if ((g.epi & EPI_GELU) && !aligned_to(g.C2, 8)) return false;
  return true;
}

hipError_t launch_gemm(Dtype dt, const GemmArgs& g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
  if (gemm_uses_mfma(dt, g)) {
    // tile choice: the largest tile that still gives every CU work
    long t256 = (long)((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch;
    long t2x1 = (long)((g.M + 255) / 256) * ((g.N + 127) / 128) * g.batch;
    if (t256 >= 256) return launch_mfma_layout<256, 256>(g, st);
    if (t2x1 >= 256) return launch_mfma_layout<256, 128>(g, st);
    return launch_mfma_layout<128, 128>(g, st);
  }
  dim3 blk(32, 8);
  dim3 grid((g.N + 31) / 32, (g.M + 7) / 8, g.batch);
  if (dt == DT_BF16)
    hipLaunchKernelGGL(gemm_plain_kernel<bf16>, grid, blk, 0, st, g);
  else
    hipLaunchKernelGGL(gemm_plain_kernel<float>, grid, blk, 0, st, g);
  return hipGetLastError();
}

}  // namespace dapple
