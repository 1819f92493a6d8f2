/*
 * dapple_kernels.h -- kernel-level entry points of the stage library.
 *
 * The forward and backward tasks of a stage (dapple_stage.h) are sequences of the
 * kernels below.  They are exported so that each can be checked against the CPU
 * oracle on its own and timed on its own; they add no functionality.  All
 * pointers are DEVICE pointers owned by the caller, `stream` is a hipStream_t
 * (NULL = default stream), work is enqueued and not waited for, the return value
 * is 0 or a negative STAGE_E_* code (see dapple_stage.h).
 * dtype: 0 = fp32, 1 = bf16 storage with fp32 accumulation.
 */
#ifndef DAPPLE_KERNELS_H
#define DAPPLE_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DAPPLE_EPI_BIAS = 1,  /* t = acc + bias[n] */
  DAPPLE_EPI_ADD = 2,   /* t += aux[m,n]  (residual branch) */
  DAPPLE_EPI_MUL = 4,   /* t *= aux[m,n]  (GELU' gate in the FFN backward) */
  DAPPLE_EPI_GELU = 8,  /* C = GELU(t), C2 = GELU'(t) */
  DAPPLE_EPI_ACC32 = 16, /* C is fp32 and C += t  (weight-gradient accumulation over
                            micro-batches, section V-B-3 of the DAPPLE paper) */
  DAPPLE_EPI_OUT32 = 32, /* C is fp32 and C = t */
  DAPPLE_EPI_AUX32 = 64, /* aux is fp32 although the product is bf16 (the unrounded residual stream) */
  DAPPLE_EPI_BSUM = 128, /* bsum[n] += sum_k B(n,k): the bias gradient (column sums of the output gradient)
                            in the launch of the weight gradient; both operands k-strided, batch 1 */
  DAPPLE_EPI_ROWDOT = 256 /* rowdot[j*M + m] = sum over the columns n in [32j, 32j+32) of C[m,n] (as stored,
                            rounded to bf16) * aux[m,n]; aux is neither added nor multiplied in.  The stage
                            backward B_s uses it on the product that makes the attention output's gradient:
                            the row sums rowsum(dctx o ctx) per head that the softmax backward needs are then
                            two of these blocks.  bf16 MFMA path only (anything else: STAGE_E_CONFIG), no other
                            epilogue than BIAS and AUX32 beside it, batch 1 */
};

/* C[m,n] = epilogue(sum_k A(m,k) B(n,k)).  A k-contiguous operand is X(r,k) =
 * X[r*ld + k]; a k-strided one is X(r,k) = X[k*ld + r].  K may be cut in segments
 * of kseg_len (0 = one segment): segment i reads A + i*segA, B + i*segB.  batch
 * (0 = 1) instances at element strides sA, sB, sC, sBias.  k_valid (0 = K): rows k
 * >= k_valid of a k-strided operand read as zero.  The linear layers of an
 * encoder layer, their data gradients and their weight gradients are all
 * instances of this product. */
typedef struct {
  const void* A;
  const void* B;
  void* C;
  void* C2;
  const void* bias;
  const void* aux;
  float* bsum;    /* DAPPLE_EPI_BSUM: fp32 [N], accumulated into */
  float* rowdot;  /* DAPPLE_EPI_ROWDOT: fp32 [ceil(N/32)][M], overwritten */
  int32_t M, N, K;
  int32_t lda, ldb, ldc, ldaux;
  int32_t a_kstrided, b_kstrided;
  int32_t kseg_len;
  int64_t segA, segB;
  int32_t batch;
  int64_t sA, sB, sC, sBias;
  int32_t k_valid;
  int32_t epi;
  int32_t tile;   /* 0 = automatic; else one configuration of the MFMA kernel, for tests and timing:
                   * 1: 256x256 tile, four-stage ring of 32-wide k-tiles; 2: 256x128, three stages of 64;
                   * 3: 128x128, two stages of 64; 4: 128x64, three stages of 64; 5: 128x128, four stages of 32
                   * (both operands k-strided; any other layout gets 3); 6: 256x128, three stages of 32 */
} dapple_gemm_desc;

/* Returns 1 if the bf16 MFMA kernel takes this problem, 0 if the plain kernel does. */
int dapple_gemm(int dtype, const dapple_gemm_desc* d, void* stream);

/* Attention of one layer.  q,k,v,ctx,dctx,dq,dk,dv: [b*s, H], head h in columns
 * [h*d, (h+1)*d), d = H / A.  lse [b,A,s] fp32: log2-domain logsumexp of the scaled
 * logits (written by fwd, read by bwd).  delta [b,A,s] fp32: scratch of bwd.
 * fwd: ctx = softmax(q k^T / sqrt(d)) v.  bwd: dq, dk, dv from dctx. */
int dapple_attention_fwd(int dtype, const void* q, const void* k, const void* v, void* ctx, float* lse,
                         int b, int s, int A, int H, void* stream);
int dapple_attention_bwd(int dtype, const void* q, const void* k, const void* v, const void* ctx,
                         const float* lse, const void* dctx, void* dq, void* dk, void* dv, float* delta,
                         int b, int s, int A, int H, void* stream);

/* y = LN(z) over the last dimension H (biased variance, eps inside the root);
 * stats[2r] = mean, stats[2r+1] = 1/sqrt(var+eps). */
int dapple_layernorm_fwd(int dtype, const void* z, const void* gamma, const void* beta, void* y,
                         float* stats, int rows, int H, float eps, void* stream);
/* dz from dy; dgamma += sum_r dy*xhat, dbeta += sum_r dy, dbias += sum_r dz (each
 * fp32 [H], NULL to skip).  partial: fp32 scratch of ceil(rows/8)*3*H elements. */
int dapple_layernorm_bwd(int dtype, const void* dy, const void* z, const float* stats, const void* gamma,
                         void* dz, float* partial, float* dgamma, float* dbeta, float* dbias, int rows,
                         int H, void* stream);
/* out[c] += sum_r X[r*ld + c]; partial: fp32 scratch of ceil(rows/64)*cols elements. */
int dapple_colsum(int dtype, const void* X, int rows, int cols, int ld, float* partial, float* out,
                  void* stream);


/* dapple_colsum for callers that cannot allocate or bring a workspace (code under HIP graph capture, serving
 * loops, harnesses that forbid hipMalloc): the same two kernels and the same summation order, bit for bit, with
 * the partial sums in an array built into the library's device code (one copy of
 * DAPPLE_COLSUM_STATIC_MAX_FLOATS floats = 4 MiB per GPU, held until the process ends).  Allocates nothing and
 * frees nothing; the array's device address is looked up on the first call on a device (a host-side query, no
 * allocation).  ceil(rows/64)*cols must not exceed DAPPLE_COLSUM_STATIC_MAX_FLOATS, else STAGE_E_CONFIG
 * (stage_last_error() says by how much) and nothing is enqueued.  X [rows, ld] and out [cols] are device
 * pointers owned by the caller as in dapple_colsum.  All calls on one GPU share the one array: calls that may
 * overlap on that GPU (different streams, no ordering between them) race; calls on one stream are safe. */
#define DAPPLE_COLSUM_STATIC_MAX_FLOATS (1 << 20)
int dapple_colsum_static(int dtype, const void* X, int rows, int cols, int ld, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif
