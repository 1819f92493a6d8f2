// C ABI of the kernel-level entry points (dapple_kernels.h): argument checks and
// forwarding to the launchers, nothing else.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/dapple_kernels.h"
#include "../../include/dapple_stage.h"
#include "kernels.h"

using namespace dapple;

// Scratch of dapple_colsum_static: the per-block partial sums of the column sum live in this array instead of a
// buffer the caller brings.  Every GPU the library runs on holds its own copy (4 MiB) at its own address until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress: the device address is
// looked up once per device and kept in scratch_ptr[], and only that pointer is ever given to a kernel.
static __device__ __align__(256) float scratch[DAPPLE_COLSUM_STATIC_MAX_FLOATS];
static std::mutex scratch_mu;
static float* scratch_ptr[64] = {};

// the current device's copy of `scratch` (looked up on the first call on that device)
static int scratch_of_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
    return set_error(STAGE_E_DEVICE, "hipGetDevice failed or device index %d out of range", dev);
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return set_error(STAGE_E_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    scratch_ptr[dev] = (float*)p;
  }
  *out = scratch_ptr[dev];
  return STAGE_OK;
}

static int dev_rc(hipError_t e) { return e == hipSuccess ? STAGE_OK : STAGE_E_DEVICE; }
static bool bad_dtype(int dt) { return dt != STAGE_DTYPE_F32 && dt != STAGE_DTYPE_BF16; }

extern "C" {

int dapple_gemm(int dtype, const dapple_gemm_desc* d, void* stream) {
  if (!d || !d->A || !d->B || !d->C) return STAGE_E_NULL;
  if (bad_dtype(dtype) || d->M < 1 || d->N < 1 || d->K < 1) return STAGE_E_CONFIG;
  if ((d->epi & DAPPLE_EPI_BIAS) && !d->bias) return STAGE_E_NULL;
  if ((d->epi & (DAPPLE_EPI_ADD | DAPPLE_EPI_MUL)) && !d->aux) return STAGE_E_NULL;
  if ((d->epi & DAPPLE_EPI_GELU) && !d->C2) return STAGE_E_NULL;
  if (d->epi & DAPPLE_EPI_BSUM) {
    if (!d->bsum) return STAGE_E_NULL;
    if (!d->a_kstrided || !d->b_kstrided || d->batch > 1) return STAGE_E_CONFIG;
  }
  if (d->epi & DAPPLE_EPI_ROWDOT) {
    if (!d->rowdot || !d->aux) return STAGE_E_NULL;
    if ((d->epi & (DAPPLE_EPI_ADD | DAPPLE_EPI_MUL | DAPPLE_EPI_GELU | DAPPLE_EPI_ACC32 | DAPPLE_EPI_OUT32)) || d->batch > 1)
      return STAGE_E_CONFIG;
  }
  GemmArgs g{};
  g.A = d->A; g.B = d->B; g.C = d->C; g.C2 = d->C2; g.bias = d->bias; g.aux = d->aux;
  g.M = d->M; g.N = d->N; g.K = d->K; g.lda = d->lda; g.ldb = d->ldb; g.ldc = d->ldc; g.ldaux = d->ldaux;
  g.a_kstrided = d->a_kstrided; g.b_kstrided = d->b_kstrided;
  g.kseg_len = d->kseg_len ? d->kseg_len : d->K; g.segA = d->segA; g.segB = d->segB;
  g.batch = d->batch ? d->batch : 1; g.sA = d->sA; g.sB = d->sB; g.sC = d->sC; g.sBias = d->sBias;
  g.k_valid = d->k_valid ? d->k_valid : d->K; g.epi = d->epi; g.tile = d->tile;
  g.m_valid = d->M; g.n_valid = d->N; g.bsum_z[0] = d->bsum;
  if (g.K % g.kseg_len) return STAGE_E_CONFIG;
  Dtype dt = dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32;
  g.rowdot = d->rowdot;
  int mfma = gemm_uses_mfma(dt, g) ? 1 : 0;
  if ((g.epi & EPI_ROWDOT) && !mfma) return STAGE_E_CONFIG;  // the plain kernel has no such epilogue
  hipError_t e = launch_gemm(dt, g, (hipStream_t)stream);
  return e == hipSuccess ? mfma : STAGE_E_DEVICE;
}

int dapple_attention_fwd(int dtype, const void* q, const void* k, const void* v, void* ctx, float* lse, int b,
                         int s, int A, int H, void* stream) {
  if (!q || !k || !v || !ctx || !lse) return STAGE_E_NULL;
  if (bad_dtype(dtype) || b < 1 || s < 1 || A < 1 || H < 1 || H % A) return STAGE_E_CONFIG;
  AttnArgs a{};
  a.q = q; a.k = k; a.v = v; a.ctx = ctx; a.lse = lse; a.b = b; a.s = s; a.A = A; a.d = H / A; a.H = H;
  return dev_rc(launch_attn_fwd(dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32, a, (hipStream_t)stream));
}

int dapple_attention_bwd(int dtype, const void* q, const void* k, const void* v, const void* ctx,
                         const float* lse, const void* dctx, void* dq, void* dk, void* dv, float* delta, int b,
                         int s, int A, int H, void* stream) {
  if (!q || !k || !v || !ctx || !lse || !dctx || !dq || !dk || !dv || !delta) return STAGE_E_NULL;
  if (bad_dtype(dtype) || b < 1 || s < 1 || A < 1 || H < 1 || H % A) return STAGE_E_CONFIG;
  AttnArgs a{};
  a.q = q; a.k = k; a.v = v; a.ctx = const_cast<void*>(ctx); a.lse = const_cast<float*>(lse); a.dctx = dctx;
  a.dq = dq; a.dk = dk; a.dv = dv; a.delta = delta; a.b = b; a.s = s; a.A = A; a.d = H / A; a.H = H;
  return dev_rc(launch_attn_bwd(dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32, a, (hipStream_t)stream));
}

static bool ln_shape_ok(int dtype, int rows, int H) {
  int vec = dtype == STAGE_DTYPE_BF16 ? 8 : 4;
  return rows >= 1 && H >= 1 && H % vec == 0 && H <= 64 * vec * 4;
}

int dapple_layernorm_fwd(int dtype, const void* z, const void* gamma, const void* beta, void* y, float* stats,
                         int rows, int H, float eps, void* stream) {
  if (!z || !gamma || !beta || !y || !stats) return STAGE_E_NULL;
  if (bad_dtype(dtype) || !ln_shape_ok(dtype, rows, H)) return STAGE_E_CONFIG;
  return dev_rc(launch_ln_fwd(dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32, z, false, gamma, beta, y, nullptr, stats, rows, H, eps,
                              (hipStream_t)stream));
}

int dapple_layernorm_bwd(int dtype, const void* dy, const void* z, const float* stats, const void* gamma, void* dz,
                         float* partial, float* dgamma, float* dbeta, float* dbias, int rows, int H, void* stream) {
  if (!dy || !z || !stats || !gamma || !dz || !partial) return STAGE_E_NULL;
  if (bad_dtype(dtype) || !ln_shape_ok(dtype, rows, H)) return STAGE_E_CONFIG;
  int nblk = 0;
  hipError_t e = launch_ln_bwd(dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32, dy, z, false, stats, gamma, dz, partial, &nblk,
                               rows, H, (hipStream_t)stream);
  if (e != hipSuccess) return STAGE_E_DEVICE;
  return dev_rc(launch_partial_reduce(partial, nblk, 3, H, dgamma, dbeta, dbias, (hipStream_t)stream));
}

int dapple_colsum(int dtype, const void* X, int rows, int cols, int ld, float* partial, float* out, void* stream) {
  if (!X || !partial || !out) return STAGE_E_NULL;
  int vec = dtype == STAGE_DTYPE_BF16 ? 8 : 4;
  if (bad_dtype(dtype) || rows < 1 || cols < 1 || cols % vec || ld % vec) return STAGE_E_CONFIG;
  return dev_rc(launch_colsum(dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32, X, rows, cols, ld, partial, out, 1, 0, 0,
                              (hipStream_t)stream));
}

int dapple_colsum_static(int dtype, const void* X, int rows, int cols, int ld, float* out, void* stream) {
  if (!X || !out) return set_error(STAGE_E_NULL, "X and out must not be NULL");
  int vec = dtype == STAGE_DTYPE_BF16 ? 8 : 4;
  if (bad_dtype(dtype) || rows < 1 || cols < 1 || cols % vec || ld % vec)
    return set_error(STAGE_E_CONFIG, "dtype, rows, cols or ld not accepted (cols and ld must be multiples of %d)", vec);
  // what the two kernels write and read: ceil(rows/64) blocks of cols partial sums (cols is a whole number of vectors)
  const size_t need = (size_t)((rows + 63) / 64) * (size_t)cols;
  if (need > (size_t)DAPPLE_COLSUM_STATIC_MAX_FLOATS)
    return set_error(STAGE_E_CONFIG, "ceil(rows/64)*cols = %zu partial sums exceed the built-in scratch of %d floats",
                     need, (int)DAPPLE_COLSUM_STATIC_MAX_FLOATS);
  float* partial = nullptr;
  int rc = scratch_of_current_device(&partial);
  if (rc != STAGE_OK) return rc;
  // every partial sum the second kernel reads is written by the first one of the same call: nothing to clear
  return dev_rc(launch_colsum(dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32, X, rows, cols, ld, partial, out, 1, 0, 0,
                              (hipStream_t)stream));
}

}  // extern "C"
