// Internal launcher interface between the host-side stage sequencer and the
// gfx950 kernels.  Plain structs and pointers; every launcher enqueues on the
// given stream and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dapple {

enum Dtype { DT_F32 = 0, DT_BF16 = 1 };

// ---------------------------------------------------------------- GEMM
// C[m,n] = epilogue( sum_k A(m,k) * B(n,k) ),  m < M, n < N, k < K.
// Operand addressing: a "k-contiguous" operand X(r,k) = X[r*ld + k]; a
// "k-strided" operand X(r,k) = X[k*ld + r].
// K may be cut in segments of kseg_len: segment s reads A + s*segA, B + s*segB
// with k running inside the segment (used to contract over [dq|dk|dv] held in
// three separate buffers).  batch: grid.z instances at strides sA, sB, sC, sBias.
enum GemmEpi {
  EPI_BIAS = 1,   // t = acc + bias[n]
  EPI_ADD = 2,    // t += aux[m,n]
  EPI_MUL = 4,    // t *= aux[m,n]
  EPI_GELU = 8,   // C = gelu(t), C2 = gelu'(t)
  EPI_ACC32 = 16,  // C is fp32 and C += t (weight-gradient accumulation)
  EPI_OUT32 = 32,  // C is fp32 and C = t
  EPI_AUX32 = 64,  // aux is fp32 (residual stream of a bf16 stage)
  EPI_BSUM = 128,  // bsum[n] += sum_k B(n,k): the bias gradient rides along with the weight gradient
  // rowdot[j*M + m] = sum over the 32 columns n of block j of C[m,n] (as stored, rounded to bf16) * aux[m,n];
  // aux is neither added nor multiplied in.  MFMA kernel only, bf16 output, batch 1.  (The attention
  // backward's delta = rowsum(dctx o ctx) per head leaves the product that makes dctx this way.)
  EPI_ROWDOT = 256
};

struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  void* C2;
  const void* bias;
  const void* aux;
  int M, N, K;
  int lda, ldb, ldc, ldaux;
  int a_kstrided, b_kstrided;
  int kseg_len;
  long segA, segB;
  int batch;
  long sA, sB, sC, sBias;
  // optional per-instance operand pointers (batch <= 4); when Az[0] / Bz[0] / Cz[0] is set
  // they replace A + z*sA / B + z*sB / C + z*sC, so unrelated products of one shape can
  // share a launch
  const void* Az[4];
  const void* Bz[4];
  void* Cz[4];
  // EPI_BSUM: fp32 [N] per instance (a NULL entry skips that instance); both operands k-strided
  float* bsum_z[4];
  float* rowdot;  // EPI_ROWDOT: fp32 [ceil(N/32)][M]
  int k_valid;  // k-strided operands: rows k >= k_valid read as zero (K itself is padded)
  int m_valid, n_valid;  // rows of A / B that exist in memory (0 = M / N); rows beyond read as zero
  int epi;
  int tile;  // 0 = automatic choice; 1..6 = a specific tile shape / ring depth (see launch_gemm)
};

hipError_t launch_gemm(Dtype dt, const GemmArgs& g, hipStream_t st);
// true when the MFMA kernel takes this problem (else the plain ALU kernel does)
bool gemm_uses_mfma(Dtype dt, const GemmArgs& g);

// ---------------------------------------------------------------- attention
// q,k,v,ctx,dq,dk,dv,dctx: [b*s, H] row-major, head h in columns [h*d, (h+1)*d).
// lse: [b, A, s] fp32, log2-domain logsumexp of the scaled logits.
// delta: [b, A, s] fp32 scratch, rowsum(dctx * ctx) per head.
// delta_blocks (may be NULL): fp32 [H/32][b*s], the same sums per block of 32 columns as EPI_ROWDOT
// of the product that made dctx leaves them; when set, the MFMA backward reads delta from there
// (a head's d/32 blocks added in ascending order) and `delta` is not touched.
// ctx32 (may be NULL): unrounded fp32 copy of ctx, written by the forward and used by the
// backward for delta -- an error in delta shifts a whole row of dS coherently, so a bf16 ctx
// there costs percents of accuracy in dq and dk although ctx itself is accurate to 2^-9.
struct AttnArgs {
  const void *q, *k, *v;
  void* ctx;
  float* ctx32;
  float* lse;
  const void* dctx;
  void *dq, *dk, *dv;
  float* delta;
  const float* delta_blocks;
  int b, s, A, d, H;
};
hipError_t launch_attn_fwd(Dtype dt, const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_bwd(Dtype dt, const AttnArgs& a, hipStream_t st);
bool attn_uses_mfma(Dtype dt, const AttnArgs& a);

// ---------------------------------------------------------------- row kernels
// y = LN(z) over the last dim (H), stats[2*r] = mean, stats[2*r+1] = rstd.  z_f32: z is fp32
// although the stage is bf16 (the residual stream is kept unrounded); y32 (may be NULL): an
// fp32 copy of y for the next residual add.
hipError_t launch_ln_fwd(Dtype dt, const void* z, bool z_f32, const void* gamma, const void* beta, void* y,
                         float* y32, float* stats, int rows, int H, float eps, hipStream_t st);
// dz = LN backward; partial[(blk*3 + {0,1,2})*H + c] = block partial sums of
// dy*xhat (dgamma), dy (dbeta), dz (bias of the linear that produced z).
// Returns the number of partial blocks through *nblk.
hipError_t launch_ln_bwd(Dtype dt, const void* dy, const void* z, bool z_f32, const float* stats,
                         const void* gamma, void* dz, float* partial, int* nblk, int rows, int H,
                         hipStream_t st);
// o_v[c] += sum over blk (ascending) of partial[(blk*nvec + v)*H + c], v < nvec <= 3;
// a NULL o_v is skipped
hipError_t launch_partial_reduce(const float* partial, int nblk, int nvec, int H, float* o0,
                                 float* o1, float* o2, hipStream_t st);
// out[c] += sum_r X[r*ld + c]  (two fixed-order stages through `partial`); nb instances at
// element strides zs_x (X) and zs_out (out); partial needs nb * ceil(rows/64) * cols floats
hipError_t launch_colsum(Dtype dt, const void* X, int rows, int cols, int ld, float* partial,
                         float* out, int nb, long zs_x, long zs_out, hipStream_t st);
// first stage of launch_colsum alone: partial[(z*nblk + blk)*PS + c], blk < *nblk = ceil(rows/64) blocks of 64 rows
hipError_t launch_colsum_partials(Dtype dt, const void* X, int rows, int cols, int ld, float* partial, int nb, long zs_x,
                                  int* nblk, int* PS_out, hipStream_t st);
// out[c] += sum over blk (ascending, in the order of launch_partial_reduce) of partial[blk*stride + c], c < cols,
// for up to 12 such jobs in one launch
struct ReduceJob {
  const float* partial;
  float* out;
  int nblk, cols;
  long stride;
};
struct ReduceJobs {
  ReduceJob j[12];
  int n;
};
hipError_t launch_reduce_jobs(const ReduceJobs& J, hipStream_t st);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
hipError_t launch_zero(void* dst, size_t bytes, hipStream_t st);

// ---------------------------------------------------------------- embedding / head
// e[r] = E_w[ids[r]] + E_p[r % s]
hipError_t launch_embed_gather(Dtype dt, const int32_t* ids, const void* Ew, const void* Ep, void* e, int rows, int s,
                               int H, int vocab, hipStream_t st);
// dEw[id] += sum over rows r with ids[r] == id (ascending r) of de[r];
// dEp[p] += sum over the b sequences of de[bi*s + p]
hipError_t launch_embed_bwd(Dtype dt, const int32_t* ids, const void* de, float* dEw, float* dEp, int b, int s, int H,
                            int vocab, hipStream_t st);
// rows_idx / tgt [np], np >= cap: the rows with target >= 0 in ascending order, at most cap of them
// (-1 / 0 in every other entry); info[0] = count, info[1] set to 1 if more than cap rows are predicted
hipError_t launch_mlm_compact(const int32_t* targets, int T, int cap, int np, int vocab, int32_t* rows_idx,
                              int32_t* tgt, int32_t* info, hipStream_t st);
// dst[i] = src[idx[i]] (zero row if idx[i] is outside [0, nsrc)); dst[idx[i]] = src[i]
hipError_t launch_gather_rows(Dtype dt, const void* src, const int32_t* idx, void* dst, int n, int H, int nsrc,
                              hipStream_t st);
hipError_t launch_scatter_rows(Dtype dt, const void* src, const int32_t* idx, void* dst, int n, int H, int ndst,
                               hipStream_t st);
// logits fp32 [n, VP] (+ bias over v < V) -> dz [n, VP], row_loss [n], loss_out[0] = loss_scale * sum(row_loss)
hipError_t launch_mlm_ce(Dtype dt, const float* logits, const void* bias, const int32_t* rows_idx, const int32_t* tgt,
                         int n, int V, int VP, float loss_scale, void* dz, float* row_loss, float* loss_out,
                         hipStream_t st);
hipError_t launch_mul(Dtype dt, const void* a, const void* b, void* c, long n, hipStream_t st);

// ---------------------------------------------------------------- weight update
// One Adam step over n parameters: g = grad_scale * G; m, v, w32 updated in fp32 (c1, c2: the
// reciprocal bias corrections 1/(1-beta1^step), 1/(1-beta2^step)); w = w32 in the stage's dtype;
// G is zeroed when zero_grads is set.  All fp32 pointers 16-byte aligned.
hipError_t launch_adam(Dtype dt, float* G, float* w32, float* m, float* v, void* w, size_t n, float lr, float beta1,
                       float beta2, float eps, float c1, float c2, float grad_scale, int zero_grads, hipStream_t st);

// ---------------------------------------------------------------- host-side plumbing shared by the C-ABI files
// records the message stage_last_error() returns and hands the code back
int set_error(int code, const char* fmt, ...);
// the compute-unit mask of a stream made by pipeline_partition_stream_create (NULL for any other stream);
// n_words receives its length in 32-bit words
const uint32_t* partition_mask_of(hipStream_t st, int* n_words);

}  // namespace dapple
