// Self-attention of one encoder layer, forward and backward, without ever
// writing the s x s probability matrix to HBM.
//
//   forward :  ctx = softmax(q k^T / sqrt(d)) v        + row logsumexp (log2 domain)
//   backward:  P = exp2(t - lse),  dP = dctx v^T,  dS = P o (dP - delta),
//              delta = rowsum(dctx o ctx),
//              dv = P^T dctx,  dq = dS k / sqrt(d),  dk = dS^T q / sqrt(d)
//
// MFMA kernels (bf16, d = 64, s % 64 == 0): a workgroup of 4 waves; each wave owns
// 32 query rows (forward, dq) or 32 key rows (dk/dv) whose fragments stay in
// registers, and streams 64-row blocks of the other side through LDS.  The
// products are oriented so that the accumulator's lane index is the row the wave
// owns: softmax statistics are then per-lane scalars, and the probabilities leave
// the accumulator already laid out as the next MFMA's operand (the contraction
// index is permuted, and the other operand is fetched from LDS with the same
// permutation through the LDS transpose read).  dq and dk/dv are two sets of
// workgroups that each recompute P: no atomics, every sum in a fixed order, so
// results are reproducible bit for bit.  Both sets go out in ONE launch (grid.z
// picks the role) with at most 256 registers per lane, so that a dq and a dk/dv
// workgroup share a compute unit: each is a chain MFMA -> softmax arithmetic ->
// MFMA with one wave per SIMD, and two of them on a SIMD fill each other's waits
// (b=4, s=512, A=16: 39 us as two launches one after the other, 29 us as one).
// delta = rowsum(dctx o ctx) must exist before either starts: the stage takes it
// from the epilogue of the product that makes dctx (delta_blocks), a caller
// without that product gets it from a small kernel of its own first.
//
// Plain kernels (any dtype and shape): one thread per output element, used by the
// fp32 configuration and by shapes the MFMA kernels do not take.
#include "device_common.h"
#include "kernels.h"

namespace dapple {

static constexpr float LOG2E = 1.4426950408889634f;

// ------------------------------------------------------------------ plain kernels
template <typename T>
__global__ void attn_fwd_plain(AttnArgs a, float scale2) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long total = (long)a.b * a.A * a.s * a.d;
  if (idx >= total) return;
  int dd = idx % a.d;
  int qi = (idx / a.d) % a.s;
  int hh = (idx / ((long)a.d * a.s)) % a.A;
  int bi = idx / ((long)a.d * a.s * a.A);
  const T* q = (const T*)a.q + ((long)bi * a.s + qi) * a.H + hh * a.d;
  const T* kb = (const T*)a.k + (long)bi * a.s * a.H + hh * a.d;
  const T* vb = (const T*)a.v + (long)bi * a.s * a.H + hh * a.d;
  float m = -INFINITY;
  for (int j = 0; j < a.s; ++j) {
    float t = 0.f;
    for (int e = 0; e < a.d; ++e) t = fmaf(to_f32(q[e]), to_f32(kb[(long)j * a.H + e]), t);
    m = fmaxf(m, t * scale2);
  }
  float l = 0.f, o = 0.f;
  for (int j = 0; j < a.s; ++j) {
    float t = 0.f;
    for (int e = 0; e < a.d; ++e) t = fmaf(to_f32(q[e]), to_f32(kb[(long)j * a.H + e]), t);
    float p = exp2f(t * scale2 - m);
    l += p;
    o = fmaf(p, to_f32(vb[(long)j * a.H + dd]), o);
  }
  ((T*)a.ctx)[((long)bi * a.s + qi) * a.H + hh * a.d + dd] = from_f32<T>(o / l);
  if (a.ctx32) a.ctx32[((long)bi * a.s + qi) * a.H + hh * a.d + dd] = o / l;
  if (dd == 0) a.lse[((long)bi * a.A + hh) * a.s + qi] = m + log2f(l);
}

template <typename T>
__global__ void attn_delta_kernel(AttnArgs a) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long total = (long)a.b * a.s * a.A;
  if (idx >= total) return;
  int hh = idx % a.A;
  long row = idx / a.A;  // bi*s + qi
  const T* o = (const T*)a.ctx + row * a.H + hh * a.d;
  const T* g = (const T*)a.dctx + row * a.H + hh * a.d;
  float t = 0.f;
  if (a.ctx32) {
    const float* o32 = a.ctx32 + row * a.H + hh * a.d;
    for (int e = 0; e < a.d; ++e) t = fmaf(o32[e], to_f32(g[e]), t);
  } else {
    for (int e = 0; e < a.d; ++e) t = fmaf(to_f32(o[e]), to_f32(g[e]), t);
  }
  int bi = row / a.s, qi = row % a.s;
  a.delta[((long)bi * a.A + hh) * a.s + qi] = t;
}

// which = 0: dq, 1: dk, 2: dv; one thread per output element
template <typename T>
__global__ void attn_bwd_plain(AttnArgs a, float scale2, float scale, int which) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long total = (long)a.b * a.A * a.s * a.d;
  if (idx >= total) return;
  int dd = idx % a.d;
  int ri = (idx / a.d) % a.s;
  int hh = (idx / ((long)a.d * a.s)) % a.A;
  int bi = idx / ((long)a.d * a.s * a.A);
  long hb = (long)bi * a.s * a.H + hh * a.d;
  const T *Q = (const T*)a.q + hb, *K = (const T*)a.k + hb, *V = (const T*)a.v + hb, *G = (const T*)a.dctx + hb;
  const float* lse = a.lse + ((long)bi * a.A + hh) * a.s;
  const float* dl = a.delta + ((long)bi * a.A + hh) * a.s;
  float acc = 0.f;
  for (int o = 0; o < a.s; ++o) {
    int qi = which == 0 ? ri : o, kj = which == 0 ? o : ri;
    float t = 0.f, dp = 0.f;
    for (int e = 0; e < a.d; ++e) {
      t = fmaf(to_f32(Q[(long)qi * a.H + e]), to_f32(K[(long)kj * a.H + e]), t);
      dp = fmaf(to_f32(G[(long)qi * a.H + e]), to_f32(V[(long)kj * a.H + e]), dp);
    }
    float p = exp2f(t * scale2 - lse[qi]);
    float ds = p * (dp - dl[qi]);
    if (which == 0) acc = fmaf(ds, to_f32(K[(long)kj * a.H + dd]), acc);
    else if (which == 1) acc = fmaf(ds, to_f32(Q[(long)qi * a.H + dd]), acc);
    else acc = fmaf(p, to_f32(G[(long)qi * a.H + dd]), acc);
  }
  T* out = (T*)(which == 0 ? a.dq : (which == 1 ? a.dk : a.dv));
  out[hb + (long)ri * a.H + dd] = from_f32<T>(which == 2 ? acc : acc * scale);
}

// ------------------------------------------------------------------ MFMA kernels
constexpr int AD = 64;  // head dimension

// A 64 x 64 bf16 block sits in LDS as 64 rows of 128 bytes with the 16-byte chunks of row
// r XOR-swizzled by aswz(r).  The same block is read two ways -- 128-bit reads along a
// row (16 lanes = 16 rows at a time) and transpose reads down the rows (32 lanes = 4 rows
// x 64 bytes at a time) -- and LDS has 64 four-byte banks, so either group must cover 256
// distinct bytes modulo 256: rows of equal parity need distinct chunks (a bijection of
// (r>>1)&7), and rows r and r+2 must land in different 64-byte halves (bit 2 of the
// swizzle = bit 1 of r).  Rotating the three bits of (r>>1)&7 right by one gives both.
__device__ __forceinline__ int aswz(int r) {
  int x = (r >> 1) & 7;
  return ((x & 1) << 2) | (x >> 1);
}

// a 64 x 64 block in flight from global memory: 2 chunks of 16 bytes per thread (256 threads)
typedef int i32x4 __attribute__((ext_vector_type(4)));
struct Block64 {
  // native vectors in named members: with the runtime's uint4 (a struct around a union) the
  // compiler kept the block in scratch memory and waited for the loads at once
  i32x4 c0, c1;
  __device__ __forceinline__ void load(const bf16* g, int ldg, int tid) {
    c0 = *(const i32x4*)(g + (long)(tid >> 3) * ldg + (tid & 7) * 8);
    c1 = *(const i32x4*)(g + (long)((tid + 256) >> 3) * ldg + (tid & 7) * 8);
  }
  __device__ __forceinline__ void store(bf16* S, int tid) const {
    int r = tid >> 3, kc = tid & 7;
    *(i32x4*)(S + r * AD + ((kc ^ aswz(r)) << 3)) = c0;
    r += 32;
    *(i32x4*)(S + r * AD + ((kc ^ aswz(r)) << 3)) = c1;
  }
};
// operand fragment, contraction index contiguous in LDS: rows r0 + (lane&31), k = 16 kk + 8 (lane>>5) + e
__device__ __forceinline__ bf16x8 frag_rows(const bf16* S, int r0, int kk, int lane) {
  int r = r0 + (lane & 31), kc = kk * 2 + (lane >> 5);
  return *(const bf16x8*)(S + r * AD + ((kc ^ aswz(r)) << 3));
}
// operand fragment, contraction index along LDS rows: column c0 + (lane&31); element e < 4 is
// LDS row k0 + 4 (lane>>5) + e, element 4 + e is LDS row k0 + 8 + 4 (lane>>5) + e -- the order
// in which a 32x32 accumulator hands its rows to a lane
__device__ __forceinline__ bf16x8 frag_cols(const bf16* S, int c0, int k0, int lane) {
  int i16 = lane & 15, g16 = (lane >> 4) & 1, h = lane >> 5;
  int r = k0 + 4 * h + (i16 >> 2);
  int col = c0 + 16 * g16 + 4 * (i16 & 3);
  const bf16* p0 = S + r * AD + (((col >> 3) ^ aswz(r)) << 3) + (col & 7);
  const bf16* p1 = S + (r + 8) * AD + (((col >> 3) ^ aswz(r + 8)) << 3) + (col & 7);
  return join8(lds_read_tr16(p0), lds_read_tr16(p1));
}
// global fragment of a row the wave owns: row r (or zeros), k = 16 kk + 8 (lane>>5) + e
__device__ __forceinline__ bf16x8 frag_global(const bf16* base, long row, bool ok, int ld, int kk, int lane) {
  if (!ok) {
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
    return z;
  }
  return *(const bf16x8*)(base + row * ld + kk * 16 + 8 * (lane >> 5));
}
// accumulator rows 16 ks .. 16 ks + 15 of a 32-row block, as the k-permuted operand
__device__ __forceinline__ bf16x8 acc_to_operand(const float (&p)[16], int ks) {
  bf16x8 f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[e] = (bf16)p[8 * ks + e];
    f[4 + e] = (bf16)p[8 * ks + 4 + e];
  }
  return f;
}

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

// delta of query row qi of sequence bi, head hh: from [b, A, s], or the head's two blocks of 32 columns
// out of [H/32][b*s]
__device__ __forceinline__ float delta_at(const AttnArgs& a, int bi, int hh, int qi) {
  if (a.delta_blocks) {
    const long T = (long)a.b * a.s, row = (long)bi * a.s + qi;
    return a.delta_blocks[(2 * hh) * T + row] + a.delta_blocks[(2 * hh + 1) * T + row];
  }
  return a.delta[((long)bi * a.A + hh) * a.s + qi];
}

// 2^x for x <= 0 as the bare v_exp_f32: the library exp2f wraps it in three more instructions that
// rescale denormal results, and a probability below 2^-126 may as well be zero
__device__ __forceinline__ float exp2_neg(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; ++v) z[v] = 0.f;
  return z;
}

// (Forward with the key blocks split over two waves per SIMD, merged at the end: 12.9 instead of 14.7 us alone, but
// the iteration gets 0.7% slower: the workgroup then fills both wave slots of its SIMDs and keeps the other streams'
// kernels off the compute unit.  One wave per SIMD it stays.)
__global__ __launch_bounds__(256) void attn_fwd_mfma(AttnArgs a, float scale2) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * AD];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * AD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5;
  const int bi = blockIdx.y / a.A, hh = blockIdx.y % a.A;
  const long hb = (long)bi * a.s * a.H + hh * AD;
  const bf16 *Q = (const bf16*)a.q + hb, *K = (const bf16*)a.k + hb, *V = (const bf16*)a.v + hb;
  const int qrow = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const bool qok = qrow < a.s;
  const int nkb = a.s / 64;
  Block64 kblk, vblk;  // the next key/value block, in flight while the current one is used
  kblk.load(K, a.H, tid);
  vblk.load(V, a.H, tid);

  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) qf[kk] = frag_global(Q, qrow, qok, a.H, kk, lane);

  float m = -INFINITY, l = 0.f;
  f32x16 o[2] = {zero16(), zero16()};  // rows d = 32 dblk + 8 blk + 4 h + e, column = the lane's query

  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    kblk.store(Ks, tid);
    vblk.store(Vs, tid);
    __syncthreads();
    {  // unconditional: the last iteration fetches its own block again (harmless, and it keeps
       // the in-flight block in registers instead of scratch)
      const int nb = kb + 1 < nkb ? kb + 1 : kb;
      kblk.load(K + (long)nb * 64 * a.H, a.H, tid);
      vblk.load(V + (long)nb * 64 * a.H, a.H, tid);
    }
    float p[2][16];
    float mx = -INFINITY;
    // All LDS reads of a phase are issued before its first MFMA (left to itself the compiler
    // reuses one register set and waits for every read in turn): the 8 key fragments, then the
    // 8 value fragments, which land while the softmax arithmetic runs.
    bf16x8 kf[2][4], vf[4][2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) kf[kb2][kk] = frag_rows(Ks, kb2 * 32, kk, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
      f32x16 sa = zero16();  // rows: key 32 kb2 + 8 blk + 4 h + e, column: query
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) sa = MFMA(kf[kb2][kk], qf[kk], sa);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[kb2][v] = sa[v] * scale2;
        mx = fmaxf(mx, p[kb2][v]);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < 2; ++db) vf[ks][db] = frag_cols(Vs, db * 32, ks * 16, lane);
    __builtin_amdgcn_sched_barrier(0);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float mn = fmaxf(m, mx);
    float alpha = exp2_neg(m - mn);
    float rs = 0.f;
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[kb2][v] = exp2_neg(p[kb2][v] - mn);
        rs += p[kb2][v];
      }
    rs += __shfl_xor(rs, 32, 64);
    l = l * alpha + rs;
    m = mn;
    // the running maximum of most rows settles after the first key blocks: skip the rescale of
    // the 32 accumulator registers when no lane of the wave needs it (alpha == 1 exactly)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 pf = acc_to_operand(p[ks >> 1], ks & 1);
#pragma unroll
      for (int db = 0; db < 2; ++db) o[db] = MFMA(vf[ks][db], pf, o[db]);
    }
  }
  if (qok) {
    float inv = 1.0f / l;
    bf16* C = (bf16*)a.ctx + hb + (long)qrow * a.H;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16)(o[db][4 * blk + e] * inv);
        *(bf16x4*)(C + db * 32 + 8 * blk + 4 * h) = ov;
        if (a.ctx32)
          *(float4*)(a.ctx32 + hb + (long)qrow * a.H + db * 32 + 8 * blk + 4 * h) =
              make_float4(o[db][4 * blk] * inv, o[db][4 * blk + 1] * inv, o[db][4 * blk + 2] * inv, o[db][4 * blk + 3] * inv);
      }
    if (h == 0) a.lse[((long)bi * a.A + hh) * a.s + qrow] = m + log2f(l);
  }
}

// dk, dv: the wave owns 32 key rows; query blocks of 64 stream through LDS
__device__ __forceinline__ void attn_dkdv_body(const AttnArgs& a, float scale2, float scale) {
  __shared__ __attribute__((aligned(16))) bf16 Qs[64 * AD];
  __shared__ __attribute__((aligned(16))) bf16 Gs[64 * AD];
  __shared__ __attribute__((aligned(16))) float Ls[64];
  __shared__ __attribute__((aligned(16))) float Ds[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5;
  const int bi = blockIdx.y / a.A, hh = blockIdx.y % a.A;
  const long hb = (long)bi * a.s * a.H + hh * AD;
  const bf16 *Q = (const bf16*)a.q + hb, *K = (const bf16*)a.k + hb, *V = (const bf16*)a.v + hb,
             *G = (const bf16*)a.dctx + hb;
  const float* lse = a.lse + ((long)bi * a.A + hh) * a.s;
  const int krow = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const bool kok = krow < a.s;

  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    kf[kk] = frag_global(K, krow, kok, a.H, kk, lane);
    vf[kk] = frag_global(V, krow, kok, a.H, kk, lane);
  }
  f32x16 dv[2] = {zero16(), zero16()}, dk[2] = {zero16(), zero16()};  // rows d, column = the lane's key
  const int nqb = a.s / 64;
  Block64 qblk, gblk;  // the next query / dctx block, in flight while the current one is used
  qblk.load(Q, a.H, tid);
  gblk.load(G, a.H, tid);
  float stat = tid < 64 ? lse[tid] : (tid < 128 ? delta_at(a, bi, hh, tid - 64) : 0.f);

  for (int qb = 0; qb < nqb; ++qb) {
    __syncthreads();
    qblk.store(Qs, tid);
    gblk.store(Gs, tid);
    if (tid < 64) Ls[tid] = stat;
    else if (tid < 128) Ds[tid - 64] = stat;
    __syncthreads();
    {  // unconditional (the last iteration fetches its own block again): keeps the block in registers
      const int nb = qb + 1 < nqb ? qb + 1 : qb;
      qblk.load(Q + (long)nb * 64 * a.H, a.H, tid);
      gblk.load(G + (long)nb * 64 * a.H, a.H, tid);
      stat = tid < 64 ? lse[nb * 64 + tid] : (tid < 128 ? delta_at(a, bi, hh, nb * 64 + tid - 64) : 0.f);
    }
#pragma unroll
    for (int qb2 = 0; qb2 < 2; ++qb2) {
      // every LDS read of a phase before its first MFMA (see attn_fwd_mfma)
      bf16x8 qf[4], gf[4], gc[2][2], qc[2][2];
      float4 L4s[4], D4s[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        qf[kk] = frag_rows(Qs, qb2 * 32, kk, lane);
        gf[kk] = frag_rows(Gs, qb2 * 32, kk, lane);
      }
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        L4s[blk] = *(const float4*)(Ls + qb2 * 32 + 8 * blk + 4 * h);
        D4s[blk] = *(const float4*)(Ds + qb2 * 32 + 8 * blk + 4 * h);
      }
      __builtin_amdgcn_sched_barrier(0);
      f32x16 sa = zero16(), dp = zero16();  // rows: query 32 qb2 + 8 blk + 4 h + e, column: key
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        sa = MFMA(qf[kk], kf[kk], sa);
        dp = MFMA(gf[kk], vf[kk], dp);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          gc[ks][db] = frag_cols(Gs, db * 32, qb2 * 32 + ks * 16, lane);
          qc[ks][db] = frag_cols(Qs, db * 32, qb2 * 32 + ks * 16, lane);
        }
      __builtin_amdgcn_sched_barrier(0);
      float p[16], ds[16];
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        float4 L4 = L4s[blk], D4 = D4s[blk];
        float Lv[4] = {L4.x, L4.y, L4.z, L4.w}, Dv[4] = {D4.x, D4.y, D4.z, D4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float pv = exp2_neg(sa[4 * blk + e] * scale2 - Lv[e]);
          p[4 * blk + e] = pv;
          ds[4 * blk + e] = pv * (dp[4 * blk + e] - Dv[e]);
        }
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 pf = acc_to_operand(p, ks), dsf = acc_to_operand(ds, ks);
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          dv[db] = MFMA(gc[ks][db], pf, dv[db]);
          dk[db] = MFMA(qc[ks][db], dsf, dk[db]);
        }
      }
    }
  }
  if (kok) {
    bf16* DK = (bf16*)a.dk + hb + (long)krow * a.H;
    bf16* DV = (bf16*)a.dv + hb + (long)krow * a.H;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        bf16x4 o1, o2;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o1[e] = (bf16)(dk[db][4 * blk + e] * scale);
          o2[e] = (bf16)dv[db][4 * blk + e];
        }
        *(bf16x4*)(DK + db * 32 + 8 * blk + 4 * h) = o1;
        *(bf16x4*)(DV + db * 32 + 8 * blk + 4 * h) = o2;
      }
  }
}

// dq: the wave owns 32 query rows; key blocks of 64 stream through LDS
__device__ __forceinline__ void attn_dq_body(const AttnArgs& a, float scale2, float scale) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * AD];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * AD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5;
  const int bi = blockIdx.y / a.A, hh = blockIdx.y % a.A;
  const long hb = (long)bi * a.s * a.H + hh * AD;
  const bf16 *Q = (const bf16*)a.q + hb, *K = (const bf16*)a.k + hb, *V = (const bf16*)a.v + hb,
             *G = (const bf16*)a.dctx + hb;
  const int qrow = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const bool qok = qrow < a.s;
  const float Lq = qok ? a.lse[((long)bi * a.A + hh) * a.s + qrow] : 0.f;

  const float Dq = qok ? delta_at(a, bi, hh, qrow) : 0.f;
  bf16x8 qf[4], gf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    qf[kk] = frag_global(Q, qrow, qok, a.H, kk, lane);
    gf[kk] = frag_global(G, qrow, qok, a.H, kk, lane);
  }
  f32x16 dq[2] = {zero16(), zero16()};  // rows d, column = the lane's query
  const int nkb = a.s / 64;
  Block64 kblk, vblk;
  kblk.load(K, a.H, tid);
  vblk.load(V, a.H, tid);

  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    kblk.store(Ks, tid);
    vblk.store(Vs, tid);
    __syncthreads();
    {  // unconditional: the last iteration fetches its own block again (harmless, and it keeps
       // the in-flight block in registers instead of scratch)
      const int nb = kb + 1 < nkb ? kb + 1 : kb;
      kblk.load(K + (long)nb * 64 * a.H, a.H, tid);
      vblk.load(V + (long)nb * 64 * a.H, a.H, tid);
    }
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
      // every LDS read of a phase before its first MFMA (see attn_fwd_mfma)
      bf16x8 kr[4], vr[4], kc[2][2];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        kr[kk] = frag_rows(Ks, kb2 * 32, kk, lane);
        vr[kk] = frag_rows(Vs, kb2 * 32, kk, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
      f32x16 sa = zero16(), dp = zero16();  // rows: key 32 kb2 + 8 blk + 4 h + e, column: query
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        sa = MFMA(kr[kk], qf[kk], sa);
        dp = MFMA(vr[kk], gf[kk], dp);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) kc[ks][db] = frag_cols(Ks, db * 32, kb2 * 32 + ks * 16, lane);
      __builtin_amdgcn_sched_barrier(0);
      float ds[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) ds[v] = exp2_neg(sa[v] * scale2 - Lq) * (dp[v] - Dq);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 dsf = acc_to_operand(ds, ks);
#pragma unroll
        for (int db = 0; db < 2; ++db) dq[db] = MFMA(kc[ks][db], dsf, dq[db]);
      }
    }
  }
  if (qok) {
    bf16* DQ = (bf16*)a.dq + hb + (long)qrow * a.H;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16)(dq[db][4 * blk + e] * scale);
        *(bf16x4*)(DQ + db * 32 + 8 * blk + 4 * h) = ov;
      }
  }
}

// delta [b, A, s] for the MFMA backward of a caller that has no product in front to leave it: one wave per row
// of dctx / ctx, a lane takes 8 consecutive columns, a head (64 columns) is 8 consecutive lanes
__global__ __launch_bounds__(256) void attn_delta_rows(AttnArgs a) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= (long)a.b * a.s) return;
  const int bi = (int)(row / a.s), qi = (int)(row % a.s);
  for (int c0 = 0; c0 < a.H; c0 += 512) {
    const int col = c0 + lane * 8;
    float t = 0.f;
    if (col < a.H) {
      const bf16x8 g = *(const bf16x8*)((const bf16*)a.dctx + row * a.H + col);
      if (a.ctx32) {
        const float4 lo = *(const float4*)(a.ctx32 + row * a.H + col), hi = *(const float4*)(a.ctx32 + row * a.H + col + 4);
        const float ov[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) t = fmaf((float)g[e], ov[e], t);
      } else {
        const bf16x8 o = *(const bf16x8*)((const bf16*)a.ctx + row * a.H + col);
#pragma unroll
        for (int e = 0; e < 8; ++e) t = fmaf((float)g[e], (float)o[e], t);
      }
    }
    t += __shfl_xor(t, 1, 64);
    t += __shfl_xor(t, 2, 64);
    t += __shfl_xor(t, 4, 64);
    if (col < a.H && (lane & 7) == 0) a.delta[((long)bi * a.A + col / AD) * a.s + qi] = t;
  }
}

// both roles in one launch: grid.z = 0 the dq workgroups, 1 the dk/dv workgroups
__global__ __launch_bounds__(256, 2) void attn_bwd_mfma(AttnArgs a, float scale2, float scale) {
  if (blockIdx.z == 0) attn_dq_body(a, scale2, scale);
  else attn_dkdv_body(a, scale2, scale);
}

// ------------------------------------------------------------------ launchers
static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

bool attn_uses_mfma(Dtype dt, const AttnArgs& a) {
  return dt == DT_BF16 && a.d == AD && a.s % 64 == 0 && a.H % 8 == 0 && al16(a.q) && al16(a.k) && al16(a.v) &&
         al16(a.ctx) && (a.dctx == nullptr || (al16(a.dctx) && al16(a.dq) && al16(a.dk) && al16(a.dv)));
}

hipError_t launch_attn_fwd(Dtype dt, const AttnArgs& a, hipStream_t st) {
  float scale2 = LOG2E / sqrtf((float)a.d);
  if (attn_uses_mfma(dt, a)) {
    dim3 grid((a.s + 127) / 128, a.b * a.A);
    hipLaunchKernelGGL(attn_fwd_mfma, grid, dim3(256), 0, st, a, scale2);
    return hipGetLastError();
  }
  long total = (long)a.b * a.A * a.s * a.d;
  dim3 grid((unsigned)((total + 255) / 256));
  if (dt == DT_BF16) hipLaunchKernelGGL(attn_fwd_plain<bf16>, grid, dim3(256), 0, st, a, scale2);
  else hipLaunchKernelGGL(attn_fwd_plain<float>, grid, dim3(256), 0, st, a, scale2);
  return hipGetLastError();
}

hipError_t launch_attn_bwd(Dtype dt, const AttnArgs& a, hipStream_t st) {
  float scale = 1.0f / sqrtf((float)a.d), scale2 = LOG2E * scale;
  hipError_t e;
  if (attn_uses_mfma(dt, a)) {
    if (!a.delta_blocks) {  // no product in front that left delta behind
      const long rows = (long)a.b * a.s;
      hipLaunchKernelGGL(attn_delta_rows, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, a);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    dim3 grid((a.s + 127) / 128, a.b * a.A, 2);
    hipLaunchKernelGGL(attn_bwd_mfma, grid, dim3(256), 0, st, a, scale2, scale);
    return hipGetLastError();
  }
  long nd = (long)a.b * a.s * a.A;
  dim3 gd((unsigned)((nd + 255) / 256));
  if (dt == DT_BF16) hipLaunchKernelGGL(attn_delta_kernel<bf16>, gd, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(attn_delta_kernel<float>, gd, dim3(256), 0, st, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  long total = (long)a.b * a.A * a.s * a.d;
  dim3 grid((unsigned)((total + 255) / 256));
  for (int which = 0; which < 3; ++which) {
    if (dt == DT_BF16) hipLaunchKernelGGL(attn_bwd_plain<bf16>, grid, dim3(256), 0, st, a, scale2, scale, which);
    else hipLaunchKernelGGL(attn_bwd_plain<float>, grid, dim3(256), 0, st, a, scale2, scale, which);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace dapple
