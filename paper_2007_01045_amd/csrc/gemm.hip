// GEMM kernels of the stage: every linear layer's forward, data-gradient and
// weight-gradient product is C = epilogue(sum_k A(m,k) B(n,k)) with either operand
// stored k-contiguous or k-strided.
//
//  * gemm_mfma_kernel: bf16 operands, fp32 accumulation on the gfx950 matrix
//    cores (v_mfma_f32_32x32x16_bf16).  256 threads = 4 waves in a 2x2 grid over a
//    BM x BN tile, k-tiles of 64 or 32, an LDS ring of 2 to 4 k-tiles filled by buffer
//    loads that write straight into LDS.  k-contiguous operands sit in LDS as [row][k]
//    and are read with 128-bit loads; k-strided operands sit as [k][rows] and are
//    read with the LDS transpose read, so no transposed copy of an activation or a
//    weight is ever made in HBM (both layouts XOR-swizzled against bank conflicts).  The MFMA is issued with the B fragment as its
//    first operand: each lane then owns 4 consecutive output columns of one
//    output row, which the epilogue stages through LDS into coalesced stores.
//  * gemm_plain_kernel: one thread per output element, fp32 accumulation in k
//    order; used for fp32 stages (the tiny configuration) and for shapes the MFMA
//    kernel does not take.
#include <type_traits>
#include <utility>

#include "device_common.h"
#include "kernels.h"

namespace dapple {

// ------------------------------------------------------------------ epilogue
template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmArgs& g, long zc, long zbias, int row, int col, float t) {
  if (g.epi & EPI_BIAS) t += to_f32(((const T*)g.bias)[zbias + col]);
  if (g.epi & (EPI_ADD | EPI_MUL)) {
    long ao = zc + (long)row * g.ldaux + col;
    float x = (g.epi & EPI_AUX32) ? ((const float*)g.aux)[ao] : to_f32(((const T*)g.aux)[ao]);
    t = (g.epi & EPI_ADD) ? t + x : t * x;
  }
  long o = zc + (long)row * g.ldc + col;
  if (g.epi & EPI_GELU) {
    float a, b;
    gelu_both(t, a, b);
    ((T*)g.C)[o] = from_f32<T>(a);
    ((T*)g.C2)[o] = from_f32<T>(b);
  } else if (g.epi & EPI_ACC32) {
    ((float*)g.C)[o] += t;
  } else if (g.epi & EPI_OUT32) {
    ((float*)g.C)[o] = t;
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
  const T* A = g.Az[0] ? (const T*)g.Az[z] : (const T*)g.A + z * g.sA;
  const T* B = g.Bz[0] ? (const T*)g.Bz[z] : (const T*)g.B + z * g.sB;
  if (g.Cz[0]) {
    g.C = g.Cz[z];
    g.sC = 0;
  }
  float acc = 0.f, bsum = 0.f;
  int nseg = g.K / g.kseg_len;
  for (int s = 0; s < nseg; ++s) {
    const T* As = A + s * g.segA;
    const T* Bs = B + s * g.segB;
    for (int k = 0; k < g.kseg_len; ++k) {
      if (k >= g.k_valid) break;
      float a = row < g.m_valid ? to_f32(g.a_kstrided ? As[(long)k * g.lda + row] : As[(long)row * g.lda + k]) : 0.f;
      float b = col < g.n_valid ? to_f32(g.b_kstrided ? Bs[(long)k * g.ldb + col] : Bs[(long)col * g.ldb + k]) : 0.f;
      acc = fmaf(a, b, acc);
      bsum += b;
    }
  }
  if ((g.epi & EPI_BSUM) && row == 0) {
    float* bs = z == 0 ? g.bsum_z[0] : (z == 1 ? g.bsum_z[1] : (z == 2 ? g.bsum_z[2] : g.bsum_z[3]));
    if (bs) bs[col] += bsum;
  }
  epilogue_store<T>(g, z * g.sC, z * g.sBias, row, col, acc);
}

// ------------------------------------------------------------------ MFMA kernel
constexpr unsigned BUF_RSRC_FLAGS = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)

typedef __attribute__((__vector_size__(4 * sizeof(int)))) int int4v;

// One operand's [R x BK] tile of a k-step in LDS (BK = 64 or 32), filled by buffer loads that
// write straight into LDS (16 bytes per lane, 1 KiB contiguous per wave
// instruction; out-of-range offsets read as zero, so ragged edges need no
// branches) and read back as MFMA fragments.
//   k-contiguous operand: LDS [row][BK/8 chunks of 16 B], chunk' = chunk ^ rswz(row)
//                         (BK = 64: (row >> 1) & 7; BK = 32: (row >> 2) & 3 -- in both cases the 16 rows a
//                         group of 16 lanes reads spread over all 16 sixteen-byte slots of a 256-byte bank row)
//   k-strided operand:    LDS [k][R/8 chunks],         chunk' = chunk ^ kswz(k)
// LDS has 64 banks of 4 bytes: a 128-bit read is served 16 lanes at a time and a
// 64-bit (transpose) read 32 lanes at a time, each group needing 256 distinct
// bytes modulo 256.  The swizzles give exactly that (measured: 5 and 2.6 clocks
// per wave instruction against 8 and 8 unswizzled); they are applied on the global
// side (which chunk a lane fetches), since the LDS side of a direct load is fixed
// to lane order.
//
// A wave issues one instruction every few clocks, and a k-step of a 64x64 wave tile is
// only 16 MFMAs: the loop is bound by instruction issue unless everything around the
// MFMAs is a handful of instructions.  So every per-lane address is computed once,
// before the loop (global side: voff; LDS side: FragAddr), the ring slot enters as an
// instruction immediate (the k-loop is unrolled over the ring), and the global cursor
// is a buffer resource in scalar registers that advances by two scalar adds per k-step.
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant expression
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <int R, bool KS, int NW, int BK>
struct OperandTile {
  static_assert(BK == 64 || BK == 32, "k-tiles of 64 or 32");
  static constexpr int CH = BK / 8;                   // 16-byte chunks per row of a k-contiguous tile
  static constexpr int NI = R * CH / (64 * NW);       // load instructions per wave per k-tile
  static constexpr int LDS_ELEMS = R * BK;
  static constexpr int LDS_BYTES = LDS_ELEMS * 2;
  static_assert(R * CH % (64 * NW) == 0, "tile rows must split evenly over the waves");
  int voff[NI];  // per-lane byte offset of each load inside the k-tile's slab

  // chunk swizzle of row `row` of a k-contiguous tile
  static __device__ __forceinline__ int rswz(int row) { return BK == 64 ? (row >> 1) & 7 : (row >> 2) & 3; }

  // chunk swizzle of k row k of a k-strided tile: rows of 256 B or more rotate by 64 B per
  // row (4 rows cover 256 B); rows of 128 B alternate halves every second row
  static __device__ __forceinline__ int kswz(int k) { return R >= 128 ? (k & 3) << 2 : ((k >> 1) & 1) << 2; }

  // A wave loads NI consecutive 1 KiB chunks of the tile.  The instruction's immediate offset is
  // added to the global AND to the LDS address, so the loads of a group of up to four chunks share
  // one M0 (the LDS base) and differ in the immediate; the lane offsets are compensated
  // (voff_j - 1024 j) and, to stay non-negative, shifted by BIAS, which the kernel takes out of
  // the buffer's base and adds to its record count.
  static constexpr int BIAS = 3072;
  static constexpr int GROUP = NI < 4 ? NI : 4;
  static_assert(NI % GROUP == 0 && (GROUP == 2 || GROUP == 4), "a wave loads 2, 4 or 8 chunks per operand");
  __device__ __forceinline__ void init(int ld, int r0, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      int pos = (wave * NI + j) * 64 + lane;
      if (!KS) {
        int row = pos / CH, kc = (pos % CH) ^ rswz(row);
        voff[j] = ((r0 + row) * ld + kc * 8) * 2;
      } else {
        int krow = pos / (R / 8), c = (pos % (R / 8)) ^ kswz(krow);
        voff[j] = (krow * ld + r0 + c * 8) * 2;
      }
      voff[j] += BIAS - (j % GROUP) * 1024;
    }
  }
  // Request one k-step's slab.  rs: buffer resource whose base is the slab's first element minus
  // BIAS bytes and whose num_records is the number of valid bytes from the slab's first element
  // plus BIAS (BIAS itself = nothing to read); LDS_OFF: byte offset of the tile in LDS (ring slot
  // and operand; a constant); wave_off = wave * NI * 1024.  Issued from inline assembly on
  // purpose: through the compiler builtin every LDS read that follows waits for ALL outstanding
  // loads (the compiler cannot tell the ring slots apart), which would undo the multi-stage
  // pipeline.  The kernel keeps its own count instead (s_waitcnt vmcnt(n) before the barrier).
  static constexpr int NGROUPS = NI / GROUP;
  // one group (G0 = its first chunk) of the k-tile's requests
  template <int LDS_OFF, int G0>
  __device__ __forceinline__ void load_group(int4v rs, int wave_off) const {
    // uniform already; this only tells the compiler so (no instruction when it is in SGPRs)
    rs[0] = __builtin_amdgcn_readfirstlane(rs[0]);
    rs[1] = __builtin_amdgcn_readfirstlane(rs[1]);
    rs[2] = __builtin_amdgcn_readfirstlane(rs[2]);
    rs[3] = (int)BUF_RSRC_FLAGS;
    wave_off = __builtin_amdgcn_readfirstlane(wave_off);
    // Two hazards the hardware does not interlock and the compiler cannot see inside an asm
    // block (CDNA3 ISA guide, manually inserted wait states): a scalar write of the resource
    // registers needs 5 wait states before a vector-memory instruction reads them (the compiler
    // assembles the 4-register tuple right before the block: s_nop 4), and a scalar write of M0
    // needs 1 before the LDS-direct load that uses it (s_nop 0).  One block per group, so that
    // nothing the compiler emits can come between the M0 write and its loads.
    if constexpr (GROUP == 4) {
      asm volatile(
          "s_nop 4\n\ts_add_u32 m0, %0, %1\n\ts_nop 0\n\t"
          "buffer_load_dwordx4 %2, %6, 0 offen lds\n\t"
          "buffer_load_dwordx4 %3, %6, 0 offen offset:1024 lds\n\t"
          "buffer_load_dwordx4 %4, %6, 0 offen offset:2048 lds\n\t"
          "buffer_load_dwordx4 %5, %6, 0 offen offset:3072 lds"
          :
          : "s"(wave_off), "i"(LDS_OFF + G0 * 1024), "v"(voff[G0]), "v"(voff[G0 + 1]), "v"(voff[G0 + 2]),
            "v"(voff[G0 + 3]), "s"(rs)
          : "memory", "m0", "scc");
    } else {
      asm volatile(
          "s_nop 4\n\ts_add_u32 m0, %0, %1\n\ts_nop 0\n\t"
          "buffer_load_dwordx4 %2, %4, 0 offen lds\n\t"
          "buffer_load_dwordx4 %3, %4, 0 offen offset:1024 lds"
          :
          : "s"(wave_off), "i"(LDS_OFF + G0 * 1024), "v"(voff[G0]), "v"(voff[G0 + 1]), "s"(rs)
          : "memory", "m0", "scc");
    }
  }
  template <int LDS_OFF>
  __device__ __forceinline__ void load(int4v rs, int wave_off) const {
    static_for<NGROUPS>([&](auto G) { load_group<LDS_OFF, decltype(G)::value * GROUP>(rs, wave_off); });
  }
};

// LDS byte addresses of a lane's MFMA fragments, relative to the operand's tile:
// rows w0 + 32*blk + (lane & 31), k = kk*16 + 8*(lane>>5) + 0..7.  Everything that depends
// on blk, kk or the ring slot beyond these few registers is an instruction immediate.
template <int R, bool KS, int NB, int BK>
struct FragAddr {
  static constexpr int KSTEPS = BK / 16;
  unsigned a[KS ? NB : KSTEPS];
  __device__ __forceinline__ void init(int w0, int lane) {
    if (!KS) {
      int r = lane & 31, sw = OperandTile<R, KS, 4, BK>::rswz(r);  // w0 is a multiple of 32: the swizzle sees lane bits only
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) a[kk] = (unsigned)((w0 + r) * (BK * 2) + (((kk * 2 + (lane >> 5)) ^ sw) << 4));
    } else {
      int i16 = lane & 15, g16 = (lane >> 4) & 1, h = lane >> 5;
      int krow = 8 * h + (i16 >> 2);
      int sw = OperandTile<R, KS, 4, BK>::kswz(i16 >> 2);  // depends on krow & 3 only
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        int col = w0 + 32 * b + 16 * g16 + 4 * (i16 & 3);
        a[b] = (unsigned)((krow * R + (((col >> 3) ^ sw) << 3) + (col & 7)) * 2);
      }
    }
  }
  // OFF: byte offset of the operand's tile in LDS (a constant)
  template <int OFF, int BLK, int KK>
  __device__ __forceinline__ bf16x8 get(const unsigned char* smem) const {
    if (!KS) {
      return *(const bf16x8*)(smem + a[KK] + (OFF + BLK * 32 * BK * 2));
    } else {
      const bf16* p = (const bf16*)(smem + a[BLK] + (OFF + KK * 16 * R * 2));
      return join8(lds_read_tr16(p), lds_read_tr16(p + 4 * R));
    }
  }
};

// sum over each group of 8 consecutive lanes, in every lane of the group, as a fixed tree: lane pairs, pairs of
// pairs (both inside a quad), then the two quads (the mirror image within the half row) -- cross-lane operands of
// the adds themselves, no trip through LDS
__device__ __forceinline__ float sum8(float v) {
  auto dpp = [](float x, auto CTRL) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(CTRL)::value, 0xF, 0xF, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
  v += dpp(v, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
  v += dpp(v, std::integral_constant<int, 0x141>{});  // row_half_mirror
  return v;
}

template <int BM, int BN, int WGM, int WGN, int NS, bool AKS, bool BKS, int BK>
struct GemmTile {
  static constexpr int NW = WGM * WGN, NT = 64 * NW;
  static constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
  typedef OperandTile<BM, AKS, NW, BK> TA;
  typedef OperandTile<BN, BKS, NW, BK> TB;
  static constexpr int STAGE_ELEMS = TA::LDS_ELEMS + TB::LDS_ELEMS;
  static constexpr int EPI_LD = WN + 4;  // fp32 staging row
  static constexpr size_t MAIN_BYTES = NS * (size_t)STAGE_ELEMS * sizeof(bf16);
  static constexpr int LOADS_PER_TILE = TA::NI + TB::NI;  // per wave
  static constexpr size_t EPI_BYTES = (size_t)NW * 32 * EPI_LD * sizeof(float);
  static constexpr size_t LDS_BYTES = MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES;
};

// CS: the variant that can also sum B over k (EPI_BSUM)
template <int BM, int BN, int WGM, int WGN, int NS, bool AKS, bool BKS, int BK, bool CS>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  typedef GemmTile<BM, BN, WGM, WGN, NS, AKS, BKS, BK> CFG;
  typedef typename CFG::TA TA;
  typedef typename CFG::TB TB;
  constexpr int MI = CFG::MI, NI = CFG::NI;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WGN) * CFG::WM, wn0 = (wave % WGN) * CFG::WN;

  // Tile index.  Consecutive workgroups land on different XCDs (round-robin over 8), and
  // each XCD has its own L2.  Cut the tile grid into pm x pn = 8 rectangles, one per XCD,
  // so that the A and B panels an XCD touches are as few as possible and are reused by
  // all its tiles out of its L2; inside a rectangle walk column-blocks of 4 tiles.
  int tm, tn;
  {
    const int bid = blockIdx.x;
    const int ntiles = tiles_m * tiles_n;
    int pm = 0, best = 1 << 30;
#pragma unroll
    for (int c = 1; c <= 8; c <<= 1) {
      int pn = 8 / c;
      if (tiles_m % c == 0 && tiles_n % pn == 0) {
        int cost = (tiles_m / c) * BM + (tiles_n / pn) * BN;
        if (cost < best) { best = cost; pm = c; }
      }
    }
    if (pm == 0 || (ntiles & 7)) {
      tm = bid / tiles_n;
      tn = bid % tiles_n;
    } else {
      const int pn = 8 / pm, rm = tiles_m / pm, rn = tiles_n / pn;
      const int xcd = bid & 7, local = bid >> 3;
      const int lm = local % rm, ln = local / rm;   // walk down a column of the rectangle first
      tm = (xcd / pn) * rm + lm;
      tn = (xcd % pn) * rn + ln;
    }
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int z = blockIdx.z;

  // (the per-instance pointers are picked with constant indices: a variable index would move the whole
  // argument struct to scratch memory, and with it every value the k-loop derives from it out of scalar registers)
  auto pick = [&](auto& arr) { return z == 0 ? arr[0] : (z == 1 ? arr[1] : (z == 2 ? arr[2] : arr[3])); };
  const bf16* Ab = g.Az[0] ? (const bf16*)pick(g.Az) : (const bf16*)g.A + z * g.sA;
  const bf16* Bb = g.Bz[0] ? (const bf16*)pick(g.Bz) : (const bf16*)g.B + z * g.sB;
  void* const Cb = g.Cz[0] ? pick(g.Cz) : g.C;
  const int nk = g.K / BK;
  const int tiles_per_seg = g.kseg_len / BK;
  // bytes of one segment of each operand that may be read (beyond: zero)
  const long a_ext =
      AKS ? ((long)(g.k_valid - 1) * g.lda + g.m_valid) * 2 : ((long)(g.m_valid - 1) * g.lda + g.kseg_len) * 2;
  const long b_ext =
      BKS ? ((long)(g.k_valid - 1) * g.ldb + g.n_valid) * 2 : ((long)(g.n_valid - 1) * g.ldb + g.kseg_len) * 2;

  TA ta;
  TB tb;
  ta.init(g.lda, m0, wave, lane);
  tb.init(g.ldb, n0, wave, lane);
  FragAddr<BM, AKS, MI, BK> fa;
  FragAddr<BN, BKS, NI, BK> fb;
  fa.init(wm0, lane);
  fb.init(wn0, lane);
  const int wave_off_a = wave * TA::NI * 1024, wave_off_b = wave * TB::NI * 1024;

  // Global cursors, all in scalar registers: one buffer resource per operand whose base is
  // the first element of the next k-step's slab and whose num_records is what may still be
  // read from there.  A k-step forward is base += step, records -= step; at the end of a
  // K segment the base jumps to the next segment and the records start over.
  const int a_step = AKS ? BK * g.lda * 2 : BK * 2, b_step = BKS ? BK * g.ldb * 2 : BK * 2;
  const long a_jump = g.segA * 2 - (long)(tiles_per_seg - 1) * a_step;
  const long b_jump = g.segB * 2 - (long)(tiles_per_seg - 1) * b_step;
  int4v ars, brs;
  auto set_base = [](int4v& rs, uint64_t p) {
    rs[0] = (int)(uint32_t)p;
    rs[1] = (int)(uint32_t)(p >> 32);  // a device address has no bits above 47: stride and swizzle fields stay 0
  };
  auto get_base = [](const int4v& rs) { return ((uint64_t)(uint32_t)rs[1] << 32) | (uint32_t)rs[0]; };
  set_base(ars, (uint64_t)Ab - TA::BIAS);
  set_base(brs, (uint64_t)Bb - TB::BIAS);
  ars[0] = __builtin_amdgcn_readfirstlane(ars[0]);
  ars[1] = __builtin_amdgcn_readfirstlane(ars[1]);
  brs[0] = __builtin_amdgcn_readfirstlane(brs[0]);
  brs[1] = __builtin_amdgcn_readfirstlane(brs[1]);
  // record counts carry the operand tiles' BIAS (see OperandTile); BIAS alone = nothing readable
  const int a_rec0 = (int)a_ext + TA::BIAS, b_rec0 = (int)b_ext + TB::BIAS;
  ars[2] = __builtin_amdgcn_readfirstlane(a_rec0);
  brs[2] = __builtin_amdgcn_readfirstlane(b_rec0);
  ars[3] = brs[3] = (int)BUF_RSRC_FLAGS;
  // Branch-free on purpose: with control flow inside the k-loop the accumulators get
  // copied between register files at every merge point.
  int seg_left = tiles_per_seg, tiles_left = nk;
  auto advance = [&]() {
    --seg_left;
    --tiles_left;
    const bool cross = seg_left == 0, more = tiles_left > 0;
    set_base(ars, get_base(ars) + (uint64_t)(cross ? a_jump : (long)a_step));
    set_base(brs, get_base(brs) + (uint64_t)(cross ? b_jump : (long)b_step));
    // past the last k-tile the cursor reads nothing: such a request fills its slot with zeros
    ars[2] = more ? (cross ? a_rec0 : max(ars[2] - a_step, (int)TA::BIAS)) : (int)TA::BIAS;
    brs[2] = more ? (cross ? b_rec0 : max(brs[2] - b_step, (int)TB::BIAS)) : (int)TB::BIAS;
    seg_left = cross ? tiles_per_seg : seg_left;
  };
  // request the next k-tile into ring slot S
  auto issue_loads = [&](auto S) {
    constexpr int off = decltype(S)::value * CFG::STAGE_ELEMS * 2;
    ta.template load<off>(ars, wave_off_a);
    tb.template load<off + TA::LDS_BYTES>(brs, wave_off_b);
    advance();
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Software pipeline.  Global->LDS: a k-tile is requested NS-1 iterations before it is
  // used, as soon as every wave has left the ring slot it goes to.  LDS->registers: the
  // fragments of k-step kk+1 are requested before the MFMAs of k-step kk are issued (two
  // fragment sets), so the matrix cores wait for an LDS round trip only once per tile.
  struct Frags {
    bf16x8 a[MI], b[NI];
  };
  constexpr int KSTEPS = BK / 16;
  static_assert(KSTEPS % 2 == 0, "the two fragment sets alternate over an even number of k-steps");

  // The loop runs whole turns of the ring: K is padded to a multiple of NS k-tiles with
  // tiles that read nothing (zeros in LDS add nothing), and every iteration requests a tile,
  // so the count of requests in flight is the same in every iteration.
  // vmcnt(N): at most N of this wave's requests still in flight; requests complete in order,
  // so N = (NS - 2) * LOADS_PER_TILE means "tile kt has landed"
  constexpr int INFLIGHT = (NS - 2) * CFG::LOADS_PER_TILE;
  static_assert(INFLIGHT < 64, "vmcnt is a 6-bit counter");
  // ... and lgkmcnt(0): this wave's LDS reads of the previous tile must have EXECUTED, not just
  // been issued, before the barrier lets other waves refill that slot (a request that reads
  // nothing delivers its zeros within a few clocks)
  constexpr int WAIT_TILE = (INFLIGHT & 15) | ((INFLIGHT >> 4) << 14) | 0x0070;  // expcnt: no wait
  static_for<NS - 1>([&](auto T) { issue_loads(T); });
  // The k-steps are rotated by one against the tiles: the MFMAs of a tile's LAST k-step are issued after the
  // barrier that opens the next tile (their fragments were read before it).  Everything else a tile needs --
  // the LDS reads of the next k-step's fragments, the requests for the tile NS - 1 ahead, the cursor arithmetic
  // -- is cut in pieces and placed BETWEEN the MFMAs of a k-step in a fixed order (nothing may be moved across
  // the fences): a wave issues an instruction every few clocks while an MFMA holds the matrix pipe for 32, so
  // in the shadow of each MFMA there is room for a few other instructions and the pipe never waits for them.
  // The very first rotated step multiplies zeros.
  Frags f0, f1;
  static_for<MI>([&](auto I) { f1.a[decltype(I)::value] = bf16x8{}; });
  static_for<NI>([&](auto J) { f1.b[decltype(J)::value] = bf16x8{}; });
  constexpr int GA = TA::NGROUPS, GB = TB::NGROUPS, EXTRA = GA + GB + 1;  // request groups of A, of B, the cursor step
  constexpr int NFRAG = MI + NI, NM = MI * NI;
  // step J of tile S: the MFMAs of `use`; between them the reads of `fill` (the fragments of k-step J of tile S,
  // in the order the next step's MFMAs need them: a0, b0 .. b_NI-1, a1 ..) and this step's share of the requests
  // for the tile that goes to ring slot SN
  // EPI_BSUM: bsum[n] += sum_k B(n,k) for this tile's columns, by the workgroups of the first tile row (tm == 0)
  // and there by the waves that hold the tile's first rows: one more MFMA per column block and k-step with an
  // A fragment of ones -- every row of its result is the column sum, exact products, fp32 adds in k order.
  // The matrix pipe has the room (the products wait for the global -> LDS path), and the column sums of the
  // output gradient need no pass of their own over it.
  f32x16 csum[CS ? NI : 1];
#pragma unroll
  for (int j = 0; j < (CS ? NI : 1); ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) csum[j][v] = 0.f;
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (bf16)1.0f;
  float* const bsum_ptr = CS ? pick(g.bsum_z) : nullptr;
  const bool do_cs = CS && (g.epi & EPI_BSUM) && tm == 0 && wm0 == 0 && bsum_ptr != nullptr;
  auto step = [&](const Frags& use, Frags& fill, auto S, auto SN, auto J, auto WCS) {
    constexpr int off = decltype(S)::value * CFG::STAGE_ELEMS * 2, offn = decltype(SN)::value * CFG::STAGE_ELEMS * 2;
    constexpr int j = decltype(J)::value;
    constexpr int e0 = j * EXTRA / KSTEPS, e1 = (j + 1) * EXTRA / KSTEPS, P = NFRAG + (e1 - e0);
    static_for<NM>([&](auto Q) {
      constexpr int q = decltype(Q)::value, mi = q / NI, ni = q % NI;
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(use.b[ni], use.a[mi], acc[mi][ni], 0, 0, 0);
      if constexpr (decltype(WCS)::value && mi == 0)
        csum[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(use.b[ni], ones, csum[ni], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int p0 = q * P / NM, p1 = (q + 1) * P / NM;
      static_for<p1 - p0>([&](auto D) {
        constexpr int p = p0 + decltype(D)::value;
        if constexpr (p == 0) {
          fill.a[0] = fa.template get<off, 0, j>(smem);
        } else if constexpr (p <= NI) {
          fill.b[p - 1] = fb.template get<off + TA::LDS_BYTES, p - 1, j>(smem);
        } else if constexpr (p < NFRAG) {
          fill.a[p - NI] = fa.template get<off, p - NI, j>(smem);
        } else {
          constexpr int e = e0 + (p - NFRAG);
          if constexpr (e < GA) ta.template load_group<offn, e * TA::GROUP>(ars, wave_off_a);
          else if constexpr (e < GA + GB) tb.template load_group<offn + TA::LDS_BYTES, (e - GA) * TB::GROUP>(brs, wave_off_b);
          else advance();
        }
      });
      if constexpr (p1 > p0) __builtin_amdgcn_sched_barrier(0);
    });
  };
  const int turns = (nk + NS - 1) / NS;
  auto main_loop = [&](auto WCS) {
    for (int t = 0; t < turns; ++t) {
      static_for<NS>([&](auto S) {
        typedef std::integral_constant<int, (decltype(S)::value + NS - 1) % NS> SN;
        __builtin_amdgcn_sched_barrier(0);  // no LDS read of the previous tile may sink below the barrier
        __builtin_amdgcn_s_waitcnt(WAIT_TILE);
        __builtin_amdgcn_s_barrier();  // every wave's part of this tile is in LDS; the previous tile's slot is free
        asm volatile("" ::: "memory");  // ... and no LDS read of this tile may be hoisted above it
        static_for<KSTEPS / 2>([&](auto H) {
          constexpr int kk = 2 * decltype(H)::value;
          step(f1, f0, S, SN{}, std::integral_constant<int, kk>{}, WCS);      // MFMAs of k-step kk - 1 (the previous tile's last when kk == 0)
          step(f0, f1, S, SN{}, std::integral_constant<int, kk + 1>{}, WCS);
        });
      });
    }
    // the last k-step of the last tile
    static_for<NM>([&](auto Q) {
      constexpr int q = decltype(Q)::value, mi = q / NI, ni = q % NI;
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.b[ni], f1.a[mi], acc[mi][ni], 0, 0, 0);
      if constexpr (decltype(WCS)::value && mi == 0)
        csum[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.b[ni], ones, csum[ni], 0, 0, 0);
    });
  };
  // (two copies of the loop under one uniform branch, none inside it)
  if constexpr (CS) {
    if (do_cs) main_loop(std::true_type{});
    else main_loop(std::false_type{});
  } else {
    main_loop(std::false_type{});
  }
  if constexpr (CS) {
    // every row of csum holds the column sums: the lanes of row 0 add them to bsum (one workgroup per column
    // range does, so the add needs no atomic)
    if (do_cs && (lane & 31) == 0) {
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int col = n0 + wn0 + 32 * j + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (col < g.N) bsum_ptr[col] += csum[j][v];
        }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // the tail requests (they read nothing) must be done before LDS is reused
  // The residual / gate operand of the epilogue is requested HERE, before the workgroup's last barrier and the
  // staging of the accumulators through LDS, so that its latency (up to a few microseconds when it comes from
  // HBM) passes behind them instead of being waited for once per 32-row block.  Only for the 128-row tiles: larger
  // ones would need more registers than the accumulators leave.  (The fp32 C of an accumulating product is NOT
  // requested early: measured, that costs 3 us per launch more than it hides, like every other early read of C.)
  const long zc = g.Cz[0] ? 0 : z * g.sC, zbias = z * g.sBias;
  constexpr int C4 = CFG::WN / 4;             // float4 per staged row
  constexpr int NIT = 32 * C4 / 64;           // float4 per lane per 32-row block
  constexpr int HB = NIT > 8 ? 8 : NIT;       // processed HB at a time
  constexpr bool PRE = !CS && MI * NIT <= 16;   // (the column-sum variant serves accumulating products only)
  const int epi = g.epi;
  // (native vectors: arrays of the runtime's float4, a struct around a union, stay in scratch memory; a bf16
  // operand's four values sit in the first two lanes)
  f32x4 pre[PRE ? MI : 1][PRE ? NIT : 1];
  // one 32-row block of that operand, as each lane will use it in store_block
  auto load_aux_block = [&](int i, f32x4 (&dst)[NIT]) {
    const bool interior = m0 + BM <= g.M && n0 + BN <= g.N;
    const int ldp = g.ldaux;
    const bool p32 = (epi & EPI_AUX32) != 0;
    const void* base = g.aux;
#pragma unroll
    for (int n = 0; n < NIT; ++n) {
      const int idx = n * 64 + lane, r = idx / C4, c4 = idx % C4;
      const int row = m0 + wm0 + i * 32 + r, col = n0 + wn0 + c4 * 4;
      const bool ok = interior || (row < g.M && col < g.N);
      const long o = ok ? zc + (long)row * ldp + col : zc;
      if (p32) {
        dst[n] = *(const f32x4*)((const float*)base + o);
      } else {
        typedef float f32x2 __attribute__((__vector_size__(2 * sizeof(float))));
        const f32x2 h2 = *(const f32x2*)((const bf16*)base + o);
        dst[n] = f32x4{h2[0], h2[1], 0.f, 0.f};
      }
    }
  };
  if constexpr (PRE) {
    if (epi & (EPI_ADD | EPI_MUL | EPI_ROWDOT)) {
#pragma unroll
      for (int i = 0; i < MI; ++i) load_aux_block(i, pre[i]);
    }
  }
  // every wave has read its last fragments (lgkmcnt(0)): LDS can be reused after the barrier.  The raw barrier on
  // purpose: __syncthreads() would also wait for the requests just issued.
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // epilogue: per wave, 32 output rows at a time through an fp32 LDS staging tile that
  // turns "a lane owns 4 columns of one row" into row-contiguous stores.
  // acc[i][j][v]: row = wm0 + 32 i + (lane & 31), col = wn0 + 32 j + 8 (v>>2) + 4 (lane>>5) + (v&3)
  // All LDS reads (and aux / C reads) of a half block are issued before the first use,
  // so their latencies overlap instead of adding up.
  float* stg = (float*)smem + wave * 32 * CFG::EPI_LD;
  // one 32-row block; the block index is a compile-time constant so that the
  // accumulators are always addressed statically (they must stay in registers)
  auto store_block = [&](auto I, auto FULLC) {
    constexpr int i = decltype(I)::value;
    // FULL: the whole tile lies inside the matrix, no element needs a bounds test
    constexpr bool FULL = decltype(FULLC)::value;
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 v4 = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        *(float4*)(stg + (lane & 31) * CFG::EPI_LD + j * 32 + 8 * q + 4 * (lane >> 5)) = v4;
      }
    // the staging tile is private to the wave and a wave's LDS instructions execute in
    // order: no workgroup barrier is needed (one would also wait for the stores below)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int hb = 0; hb < NIT; hb += HB) {
      float4 t[HB];
      int rows[HB], cols[HB];
#pragma unroll
      for (int u = 0; u < HB; ++u) {
        int idx = (hb + u) * 64 + lane;
        int r = idx / C4, c4 = idx % C4;
        rows[u] = m0 + wm0 + i * 32 + r;
        cols[u] = n0 + wn0 + c4 * 4;
        t[u] = *(const float4*)(stg + r * CFG::EPI_LD + c4 * 4);
      }
      {
        if (epi & EPI_BIAS) {
#pragma unroll
          for (int u = 0; u < HB; ++u)
            if (FULL || cols[u] < g.N) {
              bf16x4 bv = *(const bf16x4*)((const bf16*)g.bias + zbias + cols[u]);
              t[u].x += (float)bv[0]; t[u].y += (float)bv[1]; t[u].z += (float)bv[2]; t[u].w += (float)bv[3];
            }
        }
        if (epi & (EPI_ADD | EPI_MUL | EPI_ROWDOT)) {
          float4 xv[HB];
#pragma unroll
          for (int u = 0; u < HB; ++u) {
            if constexpr (PRE) {
              const f32x4 pv = pre[i][hb + u];
              if (epi & EPI_AUX32) {
                xv[u] = make_float4(pv[0], pv[1], pv[2], pv[3]);
              } else {
                typedef float f32x2 __attribute__((__vector_size__(2 * sizeof(float))));
                const bf16x4 b4 = __builtin_bit_cast(bf16x4, f32x2{pv[0], pv[1]});
                xv[u] = make_float4((float)b4[0], (float)b4[1], (float)b4[2], (float)b4[3]);
              }
            } else {
              bool ok = FULL || (rows[u] < g.M && cols[u] < g.N);
              long o = ok ? zc + (long)rows[u] * g.ldaux + cols[u] : zc;
              if (epi & EPI_AUX32) {
                xv[u] = *(const float4*)((const float*)g.aux + o);
              } else {
                bf16x4 b4 = *(const bf16x4*)((const bf16*)g.aux + o);
                xv[u] = make_float4((float)b4[0], (float)b4[1], (float)b4[2], (float)b4[3]);
              }
            }
          }
          if (epi & EPI_ROWDOT) {
            // a row's 32 columns of a block sit in 8 consecutive lanes (4 columns each): products of the
            // outputs as they are stored, summed over the lane's four, then over the eight lanes in a fixed tree
#pragma unroll
            for (int u = 0; u < HB; ++u) {
              const bool ok = FULL || (rows[u] < g.M && cols[u] < g.N);
              float part = (float)(bf16)t[u].x * xv[u].x + (float)(bf16)t[u].y * xv[u].y +
                           (float)(bf16)t[u].z * xv[u].z + (float)(bf16)t[u].w * xv[u].w;
              part = ok ? part : 0.f;
              part = sum8(part);
              if (ok && (lane & 7) == 0) g.rowdot[(long)(cols[u] >> 5) * g.M + rows[u]] = part;
            }
          } else {
#pragma unroll
            for (int u = 0; u < HB; ++u) {
              if (epi & EPI_ADD) {
                t[u].x += xv[u].x; t[u].y += xv[u].y; t[u].z += xv[u].z; t[u].w += xv[u].w;
              } else {
                t[u].x *= xv[u].x; t[u].y *= xv[u].y; t[u].z *= xv[u].z; t[u].w *= xv[u].w;
              }
            }
          }
        }
        if (epi & EPI_OUT32) {
#pragma unroll
          for (int u = 0; u < HB; ++u)
            if (FULL || (rows[u] < g.M && cols[u] < g.N)) *(float4*)((float*)Cb + zc + (long)rows[u] * g.ldc + cols[u]) = t[u];
        } else if (epi & EPI_ACC32) {
          float4 cv[HB];
#pragma unroll
          for (int u = 0; u < HB; ++u) {
            bool ok = FULL || (rows[u] < g.M && cols[u] < g.N);
            long o = ok ? zc + (long)rows[u] * g.ldc + cols[u] : zc;
            cv[u] = *(const float4*)((const float*)Cb + o);
          }
#pragma unroll
          for (int u = 0; u < HB; ++u)
            if (FULL || (rows[u] < g.M && cols[u] < g.N)) {
              cv[u].x += t[u].x; cv[u].y += t[u].y; cv[u].z += t[u].z; cv[u].w += t[u].w;
              *(float4*)((float*)Cb + zc + (long)rows[u] * g.ldc + cols[u]) = cv[u];
            }
        } else if (epi & EPI_GELU) {
#pragma unroll
          for (int u = 0; u < HB; ++u)
            if (FULL || (rows[u] < g.M && cols[u] < g.N)) {
              float tv[4] = {t[u].x, t[u].y, t[u].z, t[u].w};
              bf16x4 gv, gp;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                float a, b;
                gelu_both(tv[e], a, b);
                gv[e] = (bf16)a;
                gp[e] = (bf16)b;
              }
              long o = zc + (long)rows[u] * g.ldc + cols[u];
              *(bf16x4*)((bf16*)Cb + o) = gv;
              *(bf16x4*)((bf16*)g.C2 + o) = gp;
            }
        } else {
#pragma unroll
          for (int u = 0; u < HB; ++u)
            if (FULL || (rows[u] < g.M && cols[u] < g.N)) {
              bf16x4 ov;
              ov[0] = (bf16)t[u].x; ov[1] = (bf16)t[u].y; ov[2] = (bf16)t[u].z; ov[3] = (bf16)t[u].w;
              *(bf16x4*)((bf16*)Cb + zc + (long)rows[u] * g.ldc + cols[u]) = ov;
            }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  };
  auto store_tile = [&](auto FULLC) {
    store_block(std::integral_constant<int, 0>{}, FULLC);
    if constexpr (MI > 1) store_block(std::integral_constant<int, 1>{}, FULLC);
    if constexpr (MI > 2) store_block(std::integral_constant<int, 2>{}, FULLC);
    if constexpr (MI > 3) store_block(std::integral_constant<int, 3>{}, FULLC);
  };
  // interior tiles (nearly all of them) take the path without per-element bounds tests
  if (m0 + BM <= g.M && n0 + BN <= g.N) store_tile(std::true_type{});
  else store_tile(std::false_type{});
  static_assert(MI <= 4, "at most four 32-row blocks per wave");
}

// explicit instantiations (every tile shape x operand layout the launcher can pick)
#define DAPPLE_GEMM_INST(BM, BN, WGM, WGN, NS, BK)                                                               \
  template __global__ void gemm_mfma_kernel<BM, BN, WGM, WGN, NS, false, false, BK, false>(GemmArgs, int, int); \
  template __global__ void gemm_mfma_kernel<BM, BN, WGM, WGN, NS, false, true, BK, false>(GemmArgs, int, int);  \
  template __global__ void gemm_mfma_kernel<BM, BN, WGM, WGN, NS, true, false, BK, false>(GemmArgs, int, int);  \
  template __global__ void gemm_mfma_kernel<BM, BN, WGM, WGN, NS, true, true, BK, false>(GemmArgs, int, int);
DAPPLE_GEMM_INST(256, 256, 2, 2, 4, 32)
DAPPLE_GEMM_INST(256, 128, 2, 2, 3, 64)
DAPPLE_GEMM_INST(128, 128, 2, 2, 2, 64)
DAPPLE_GEMM_INST(128, 64, 2, 2, 3, 64)
DAPPLE_GEMM_INST(256, 128, 2, 2, 3, 32)
// the weight-gradient layout: 128x128 tiles with the deeper ring of 32-wide k-tiles, and the variants with the
// column sum of B
template __global__ void gemm_mfma_kernel<128, 128, 2, 2, 2, true, true, 64, true>(GemmArgs, int, int);
template __global__ void gemm_mfma_kernel<128, 64, 2, 2, 3, true, true, 64, true>(GemmArgs, int, int);
template __global__ void gemm_mfma_kernel<128, 128, 2, 2, 4, true, true, 32, true>(GemmArgs, int, int);
template __global__ void gemm_mfma_kernel<128, 128, 2, 2, 4, true, true, 32, false>(GemmArgs, int, int);
#undef DAPPLE_GEMM_INST

// ------------------------------------------------------------------ host side
template <int BM, int BN, int WGM, int WGN, int NS, bool AKS, bool BKS, int BK, bool CS = false>
static hipError_t launch_mfma(const GemmArgs& g, hipStream_t st) {
  typedef GemmTile<BM, BN, WGM, WGN, NS, AKS, BKS, BK> CFG;
  auto kern = gemm_mfma_kernel<BM, BN, WGM, WGN, NS, AKS, BKS, BK, CS>;
  // once per instantiation, whichever host thread comes first (initialisation of a function-local static is
  // thread-safe)
  static const hipError_t attr_rc = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                        (int)CFG::LDS_BYTES);
  if (attr_rc != hipSuccess) return attr_rc;
  int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  dim3 grid(tiles_m * tiles_n, 1, g.batch);
  hipLaunchKernelGGL(kern, grid, dim3(CFG::NT), CFG::LDS_BYTES, st, g, tiles_m, tiles_n);
  return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int NS, int BK = 64>
static hipError_t launch_mfma_layout(const GemmArgs& g, hipStream_t st) {
  if (g.a_kstrided) {
    return g.b_kstrided ? launch_mfma<BM, BN, WGM, WGN, NS, true, true, BK>(g, st)
                        : launch_mfma<BM, BN, WGM, WGN, NS, true, false, BK>(g, st);
  }
  return g.b_kstrided ? launch_mfma<BM, BN, WGM, WGN, NS, false, true, BK>(g, st)
                      : launch_mfma<BM, BN, WGM, WGN, NS, false, false, BK>(g, st);
}

static bool aligned_to(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

bool gemm_uses_mfma(Dtype dt, const GemmArgs& g) {
  if (dt != DT_BF16) return false;
  constexpr int BK = 64;  // every tile configuration takes K and the K segments in multiples of 64
  if (g.K < BK || g.K % BK || g.kseg_len % BK || g.K % g.kseg_len) return false;
  if (g.lda % 8 || g.ldb % 8 || g.ldc % 4 || g.N % 4) return false;
  if (g.sA % 8 || g.sB % 8 || g.sC % 4 || g.sBias % 4 || g.segA % 8 || g.segB % 8) return false;
  if (!aligned_to(g.A, 16) || !aligned_to(g.B, 16) || !aligned_to(g.C, 16)) return false;
  if (g.Az[0] || g.Bz[0] || g.Cz[0]) {
    if (g.batch > 4) return false;
    for (int z = 0; z < g.batch; ++z)
      if (!g.Az[z] || !g.Bz[z] || !g.Cz[z] || !aligned_to(g.Az[z], 16) || !aligned_to(g.Bz[z], 16) ||
          !aligned_to(g.Cz[z], 16))
        return false;
  }
  {  // the kernel counts the readable bytes of an operand segment in a 32-bit buffer field
    const int kv = g.k_valid > 0 ? g.k_valid : g.K, mv = g.m_valid > 0 ? g.m_valid : g.M, nv = g.n_valid > 0 ? g.n_valid : g.N;
    const long a_ext = g.a_kstrided ? ((long)(kv - 1) * g.lda + mv) * 2 : ((long)(mv - 1) * g.lda + g.kseg_len) * 2;
    const long b_ext = g.b_kstrided ? ((long)(kv - 1) * g.ldb + nv) * 2 : ((long)(nv - 1) * g.ldb + g.kseg_len) * 2;
    if (a_ext > 0x7fffffffL - 4096 || b_ext > 0x7fffffffL - 4096) return false;
    if ((long)BK * g.lda * 2 > 0x7fffffffL || (long)BK * g.ldb * 2 > 0x7fffffffL) return false;
  }
  if ((g.epi & (EPI_ADD | EPI_MUL | EPI_ROWDOT)) && (g.ldaux % 4 || !aligned_to(g.aux, 16))) return false;
  if ((g.epi & EPI_ROWDOT) && ((g.epi & (EPI_ADD | EPI_MUL | EPI_GELU | EPI_ACC32 | EPI_OUT32)) || g.batch != 1 ||
                               !g.rowdot || !g.aux || !aligned_to(g.rowdot, 4)))
    return false;
  if ((g.epi & EPI_BIAS) && !aligned_to(g.bias, 8)) return false;
  if ((g.epi & EPI_GELU) && !aligned_to(g.C2, 8)) return false;
  if ((g.epi & EPI_BSUM) && !(g.a_kstrided && g.b_kstrided && g.batch <= 4)) return false;
  return true;
}

hipError_t launch_gemm(Dtype dt, const GemmArgs& g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
  const bool mfma = gemm_uses_mfma(dt, g);
  if ((g.epi & EPI_ROWDOT) && !mfma) return hipErrorInvalidValue;  // only the MFMA kernel's epilogue has it
  if (mfma) {
    const long t128 = (long)((g.M + 127) / 128) * ((g.N + 127) / 128) * g.batch;
    const long t256 = (long)((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch;
    const bool tt = g.a_kstrided && g.b_kstrided;   // the weight-gradient layout
    const bool bsum = (g.epi & EPI_BSUM) != 0;      // (offered for that layout only: checked above)
    // Tile choice.  Every k-tile goes global -> LDS through the compute unit's vector cache at 64 bytes per
    // clock, and from LDS to the waves at 128 bytes per clock, against 4096 MFMA flops per clock.  A 128x128
    // tile (64x64 per wave) needs the vector cache's whole rate and 1.5 times what LDS can do (fragment reads
    // plus the arriving tiles) to keep the matrix cores busy; a 256x128 tile (128x64 per wave) 0.75 of the one
    // and 1.1 of the other; a 256x256 tile half of each, but it takes a whole compute unit.  So:
    //  - 256x256 tiles (one workgroup per unit, a four-stage ring of 32-wide k-tiles) when they alone fill the
    //    chip at least twice;
    //  - 256x128 tiles with a three-stage ring of 32-wide k-tiles (72 KB of LDS, 240 registers: two workgroups
    //    fit a unit, or one next to a workgroup of another stream's kernel) for products of at least 384
    //    128x128 tiles whose operands are not both k-strided and whose epilogue reads no second operand (this
    //    tile has no registers left to request it early).  Alone such a product is no faster than with
    //    128x128 tiles (2048 x 4096 x 1024: 23.6 against 22.4 us, one workgroup per unit); inside the stage,
    //    where the units are shared with the other streams' kernels, the iteration gains 2%.  A deeper ring
    //    (96 KB) loses more than that: the workgroup no longer fits beside another kernel's;
    //  - 128x128 tiles (two workgroups per unit) when there are at least 192 of them;
    //  - else 128x64 tiles with a three-stage ring, so that the small products of a stage (2048 x 1024 outputs)
    //    still reach every unit.
    // Weight-gradient products with at least 192 tiles take 128x128 with a four-stage ring of 32-wide k-tiles
    // in the same 64 KB of LDS: both operands are k-strided there, so a 32-deep k-tile still reads whole
    // 256-byte rows, and three tiles in flight instead of one hide the latency a two-stage ring waits for at
    // every k-tile (1024 x 4096 x 2048 in place: 43 -> 33 us).
    // GemmArgs::tile names a configuration instead (tests, timing).  Tile 5 and the column sums of B exist for
    // the weight-gradient layout only, the latter with 128-row tiles only.
    int tile = g.tile;
    if (tile == 5 && !tt) tile = 3;
    if (bsum && (tile == 1 || tile == 2 || tile == 6)) tile = 0;
    if (tile == 0) {
      if (tt && t128 >= 192) tile = 5;
      else if (!tt && t128 >= 384 && t256 < 512 && !(g.epi & (EPI_ADD | EPI_MUL))) tile = 6;
      else if (t256 >= 512 && !bsum) tile = 1;
      else tile = t128 >= 192 ? 3 : 4;
    }
    switch (tile) {
      case 1: return launch_mfma_layout<256, 256, 2, 2, 4, 32>(g, st);
      case 2: return launch_mfma_layout<256, 128, 2, 2, 3, 64>(g, st);
      case 3: return bsum ? launch_mfma<128, 128, 2, 2, 2, true, true, 64, true>(g, st)
                          : launch_mfma_layout<128, 128, 2, 2, 2, 64>(g, st);
      case 6: return launch_mfma_layout<256, 128, 2, 2, 3, 32>(g, st);
      case 5: return bsum ? launch_mfma<128, 128, 2, 2, 4, true, true, 32, true>(g, st)
                          : launch_mfma<128, 128, 2, 2, 4, true, true, 32, false>(g, st);
      default: return bsum ? launch_mfma<128, 64, 2, 2, 3, true, true, 64, true>(g, st)
                           : launch_mfma_layout<128, 64, 2, 2, 3, 64>(g, st);
    }
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
