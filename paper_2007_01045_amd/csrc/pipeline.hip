// S stages of one GPU run as a pipeline (micro-batch unit scheduling across stages, section V-C of
// the DAPPLE paper).  Host code only: it drives the stages through their public C-ABI (stage_fwd,
// stage_bwd, stage_schedule_ops) and ties them together with HIP events.
#include <hip/hip_runtime.h>

#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/dapple_pipeline.h"
#include "kernels.h"

using namespace dapple;

namespace {

std::mutex g_mask_lock;
std::map<hipStream_t, std::vector<uint32_t>> g_masks;  // partition streams and their compute-unit masks

}  // namespace

namespace dapple {
const uint32_t* partition_mask_of(hipStream_t st, int* n_words) {
  std::lock_guard<std::mutex> lk(g_mask_lock);
  auto it = g_masks.find(st);
  if (it == g_masks.end()) return nullptr;
  *n_words = (int)it->second.size();
  return it->second.data();   // map nodes do not move; the entry lives until the stream is destroyed
}
}  // namespace dapple

struct dapple_pipeline {
  int S = 0, max_M = 0;
  size_t act_bytes = 0;
  std::vector<stage_handle> stages;
  std::vector<hipStream_t> streams;
  std::vector<stage_config> cfgs;
  char* boundary = nullptr;
  // per (kind, stage, m): start and end of the task; the end event is also what dependents wait for
  std::vector<hipEvent_t> ev_start, ev_end;
  hipEvent_t ev_t0 = nullptr;
  int last_M = 0;

  size_t idx(int kind, int stage, int m) const { return ((size_t)kind * S + stage) * max_M + m; }
  // boundary b sits between stage b and stage b + 1: activation (which = 0) and gradient (which = 1)
  char* buf(int which, int b, int m) const {
    return boundary + (((size_t)which * (S - 1) + b) * max_M + m) * ((act_bytes + 255) / 256 * 256);
  }
};

extern "C" {

int pipeline_warmup_depths(int S, int M, int policy, int D, int32_t* K_out) {
  if (!K_out) return set_error(STAGE_E_NULL, "K_out must not be NULL");
  if (S < 1 || M < 1) return set_error(STAGE_E_BAD_ORDER, "S and M must be positive (S=%d, M=%d)", S, M);
  if (policy != PIPELINE_POLICY_A && policy != PIPELINE_POLICY_B) return set_error(STAGE_E_CONFIG, "unknown policy %d", policy);
  if (D <= 0 || D > M) D = M;
  for (int i = 0; i < S; ++i) {
    int k = policy == PIPELINE_POLICY_A ? S - i : 2 * (S - i) - 1;
    K_out[i] = k < D ? k : D;
  }
  return STAGE_OK;
}

int pipeline_pivot_stage(int S, int M, const double* F, const double* B) {
  if (!F || !B) return set_error(STAGE_E_NULL, "F and B must not be NULL");
  if (S < 1 || M < 1) return set_error(STAGE_E_BAD_ORDER, "S and M must be positive (S=%d, M=%d)", S, M);
  // Section IV-B-1 in prose: walking from the last stage towards the first, a stage takes the pivot from the
  // current candidate when its own steady phase, (M-1)(F_s + B_s), outweighs the candidate's steady phase plus the
  // forward and backward work of the stages strictly between the two.  That work is kept as a running sum (it
  // grows by one stage per step and starts over when the pivot moves), so every stage costs one comparison.
  int Q = S - 1;
  double steady_Q = (M - 1) * (F[Q] + B[Q]), between = 0.0;
  for (int s = S - 2; s >= 0; --s) {
    const double steady_s = (M - 1) * (F[s] + B[s]);
    if (steady_s > steady_Q + between) {
      Q = s;
      steady_Q = steady_s;
      between = 0.0;
    } else {
      between += F[s] + B[s];
    }
  }
  return Q;
}

int pipeline_latency_model(int S, int M, const double* F, const double* B, int Q, double* L_out) {
  if (!F || !B || !L_out) return set_error(STAGE_E_NULL, "F, B and L_out must not be NULL");
  if (S < 1 || M < 1) return set_error(STAGE_E_BAD_ORDER, "S and M must be positive (S=%d, M=%d)", S, M);
  if (Q < 0) Q = pipeline_pivot_stage(S, M, F, B);
  if (Q >= S) return set_error(STAGE_E_BAD_ORDER, "pivot stage %d of %d", Q, S);
  double Tw = 0.0, Te = 0.0;
  for (int s = 0; s <= Q; ++s) Tw += F[s];
  // without AllReduce the maximum over s is taken at s = 0: every backward from the pivot down to stage 0
  for (int a = 0; a <= Q; ++a) Te += B[a];
  *L_out = Tw + (M - 1) * (F[Q] + B[Q]) + Te;
  return STAGE_OK;
}

int pipeline_partition_stream_create(int part, int nparts, void** hip_stream_out) {
  if (!hip_stream_out) return set_error(STAGE_E_NULL, "hip_stream_out must not be NULL");
  if (nparts < 1 || part < 0 || part >= nparts) return set_error(STAGE_E_CONFIG, "part %d of %d", part, nparts);
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return set_error(STAGE_E_DEVICE, "hipGetDeviceProperties failed");
  const int n = prop.multiProcessorCount;
  if (nparts > n) return set_error(STAGE_E_CONFIG, "%d partitions of %d compute units", nparts, n);
  const int lo = (int)((long)part * n / nparts), hi = (int)((long)(part + 1) * n / nparts);
  std::vector<uint32_t> mask((n + 31) / 32, 0u);
  for (int i = lo; i < hi; ++i) mask[i / 32] |= 1u << (i % 32);
  hipStream_t st = nullptr;
  hipError_t e = hipExtStreamCreateWithCUMask(&st, (uint32_t)mask.size(), mask.data());
  if (e != hipSuccess) return set_error(STAGE_E_DEVICE, "hipExtStreamCreateWithCUMask failed: %s", hipGetErrorString(e));
  {
    std::lock_guard<std::mutex> lk(g_mask_lock);
    g_masks[st] = mask;
  }
  *hip_stream_out = (void*)st;
  return STAGE_OK;
}

int pipeline_partition_stream_destroy(void* hip_stream) {
  hipStream_t st = (hipStream_t)hip_stream;
  {
    std::lock_guard<std::mutex> lk(g_mask_lock);
    auto it = g_masks.find(st);
    if (it == g_masks.end()) return set_error(STAGE_E_CONFIG, "not a stream of pipeline_partition_stream_create");
    g_masks.erase(it);
  }
  if (hipStreamSynchronize(st) != hipSuccess || hipStreamDestroy(st) != hipSuccess)
    return set_error(STAGE_E_DEVICE, "hipStreamDestroy failed");
  return STAGE_OK;
}

size_t pipeline_boundary_bytes(int S, int max_M, size_t act_bytes) {
  if (S < 1 || max_M < 1) return 0;
  return (size_t)2 * (S - 1) * max_M * ((act_bytes + 255) / 256 * 256);
}

int pipeline_create(pipeline_handle* out, int S, const stage_handle* stages, void* boundary_dev, size_t boundary_bytes,
                    size_t act_bytes, int max_M) {
  if (!out || !stages) return set_error(STAGE_E_NULL, "out and stages must not be NULL");
  if (S < 1 || max_M < 1 || act_bytes == 0) return set_error(STAGE_E_CONFIG, "S, max_M and act_bytes must be positive");
  if (S > 1 && !boundary_dev) return set_error(STAGE_E_NULL, "boundary_dev must not be NULL");
  if (boundary_bytes < pipeline_boundary_bytes(S, max_M, act_bytes))
    return set_error(STAGE_E_ARENA_SMALL, "boundary buffer has %zu bytes, %zu needed", boundary_bytes,
                     pipeline_boundary_bytes(S, max_M, act_bytes));
  if ((uintptr_t)boundary_dev & 255) return set_error(STAGE_E_CONFIG, "boundary_dev must be 256-byte aligned");
  dapple_pipeline* p = new (std::nothrow) dapple_pipeline();
  if (!p) return set_error(STAGE_E_DEVICE, "out of host memory");
  p->S = S; p->max_M = max_M; p->act_bytes = act_bytes; p->boundary = (char*)boundary_dev;
  for (int i = 0; i < S; ++i) {
    void* st = nullptr;
    stage_config c;
    if (!stages[i] || stage_stream(stages[i], &st) != STAGE_OK || stage_get_config(stages[i], &c) != STAGE_OK) {
      delete p;
      return set_error(STAGE_E_NULL, "stage %d is not a live handle", i);
    }
    const size_t want = (size_t)c.micro_batch * c.seq * c.hidden * (c.dtype == STAGE_DTYPE_BF16 ? 2 : 4);
    int bad = 0;
    if (!st) bad = set_error(STAGE_E_CONFIG, "stage %d runs on the default (NULL) stream; every stage needs a stream of its own", i);
    else if (c.flags & STAGE_FLAG_DRY_RUN) bad = set_error(STAGE_E_CONFIG, "stage %d is a dry-run stage", i);
    else if (want != act_bytes) bad = set_error(STAGE_E_CONFIG, "stage %d has a boundary tensor of %zu bytes, not %zu", i, want, act_bytes);
    else if ((c.has_embedding && i != 0) || (c.has_mlm_head && i != S - 1))
      bad = set_error(STAGE_E_CONFIG, "stage %d: the embedding block belongs to the first stage, the head to the last", i);
    for (int j = 0; j < i && !bad; ++j)
      if (p->streams[j] == (hipStream_t)st) bad = set_error(STAGE_E_CONFIG, "stages %d and %d share a stream", j, i);
    if (bad) { delete p; return bad; }
    p->stages.push_back(stages[i]);
    p->streams.push_back((hipStream_t)st);
    p->cfgs.push_back(c);
  }
  const size_t n = (size_t)2 * S * max_M;
  p->ev_start.assign(n, nullptr);
  p->ev_end.assign(n, nullptr);
  bool ok = hipEventCreate(&p->ev_t0) == hipSuccess;
  for (size_t i = 0; i < n && ok; ++i)
    ok = hipEventCreate(&p->ev_start[i]) == hipSuccess && hipEventCreate(&p->ev_end[i]) == hipSuccess;
  if (!ok) {
    pipeline_destroy(p);
    return set_error(STAGE_E_DEVICE, "hipEventCreate failed");
  }
  *out = p;
  return STAGE_OK;
}

int pipeline_destroy(pipeline_handle p) {
  if (!p) return set_error(STAGE_E_NULL, "handle is NULL");
  for (hipStream_t s : p->streams) (void)hipStreamSynchronize(s);
  for (hipEvent_t e : p->ev_start) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : p->ev_end) if (e) (void)hipEventDestroy(e);
  if (p->ev_t0) (void)hipEventDestroy(p->ev_t0);
  delete p;
  return STAGE_OK;
}

int pipeline_run(pipeline_handle p, int M, const int32_t* K, int order, const void* const* xs, const void* const* dys,
                 const void* const* auxs, void* const* ys, void* const* dxs) {
  if (!p) return set_error(STAGE_E_NULL, "handle is NULL");
  const int S = p->S;
  if (M < 1 || M > p->max_M) return set_error(STAGE_E_BAD_ORDER, "M = %d outside [1, %d]", M, p->max_M);
  if (order != STAGE_ORDER_EARLY_BACKWARD && order != STAGE_ORDER_GPIPE)
    return set_error(STAGE_E_BAD_ORDER, "order must be early-backward or GPipe");
  if (order == STAGE_ORDER_EARLY_BACKWARD && !K) return set_error(STAGE_E_NULL, "K must not be NULL");
  const bool head = p->cfgs[S - 1].has_mlm_head, emb = p->cfgs[0].has_embedding;
  if (!xs || !ys || (!head && !dys) || (head && !auxs) || (!emb && !dxs))
    return set_error(STAGE_E_NULL, "a required pointer array is NULL");
  for (int m = 0; m < M; ++m)
    if (!xs[m] || !ys[m] || (!head && !dys[m]) || (head && !auxs[m]) || (!emb && !dxs[m]))
      return set_error(STAGE_E_NULL, "a device pointer of micro-batch %d is NULL", m);

  // every stage's own list (section V-C), then one global issue order: a task is enqueued once the task it
  // takes its data from has been (its event must be recorded before it can be waited for)
  std::vector<std::vector<int32_t>> lists(S);
  for (int i = 0; i < S; ++i) {
    const int k = order == STAGE_ORDER_GPIPE ? M : K[i];
    if (k < 1) return set_error(STAGE_E_BAD_ORDER, "K[%d] = %d", i, k);
    const int resident = k < M ? k : M;
    if (resident > p->cfgs[i].max_slots)
      return set_error(STAGE_E_BAD_ORDER, "stage %d would keep %d micro-batches, it has %d slots", i, resident, p->cfgs[i].max_slots);
    lists[i].resize((size_t)2 * M);
    int n = stage_schedule_ops(M, k, order, lists[i].data(), 2 * M);
    if (n != 2 * M) return n < 0 ? n : set_error(STAGE_E_BAD_ORDER, "stage %d: schedule of %d tasks", i, n);
  }
  struct Task { int stage, kind, m; };
  std::vector<Task> issue;
  issue.reserve((size_t)2 * S * M);
  {
    std::vector<char> done((size_t)2 * S * M, 0);   // [(kind * S + stage) * M + m]
    std::vector<int> pos(S, 0);
    size_t remaining = (size_t)2 * S * M;
    while (remaining) {
      bool progressed = false;
      for (int i = 0; i < S; ++i) {
        while (pos[i] < 2 * M) {
          const int32_t op = lists[i][pos[i]];
          const int kind = op > 0 ? 0 : 1, m = (op > 0 ? op : -op) - 1;
          bool ready;
          if (kind == 0) ready = i == 0 || done[((size_t)0 * S + (i - 1)) * M + m];
          else ready = i == S - 1 ? done[((size_t)0 * S + i) * M + m] != 0 : done[((size_t)1 * S + (i + 1)) * M + m] != 0;
          if (!ready) break;
          done[((size_t)kind * S + i) * M + m] = 1;
          issue.push_back({i, kind, m});
          ++pos[i];
          --remaining;
          progressed = true;
        }
      }
      if (!progressed)
        return set_error(STAGE_E_BAD_ORDER, "these warm-up depths deadlock: a later stage waits for a micro-batch an earlier "
                                            "stage only sends after a backward it is itself waiting for");
    }
  }

  auto hip_ok = [](hipError_t e) { return e == hipSuccess ? STAGE_OK : set_error(STAGE_E_DEVICE, "%s", hipGetErrorString(e)); };
  int rc = hip_ok(hipEventRecord(p->ev_t0, p->streams[0]));
  for (int i = 1; i < S && rc == STAGE_OK; ++i) rc = hip_ok(hipStreamWaitEvent(p->streams[i], p->ev_t0, 0));
  if (rc != STAGE_OK) return rc;
  p->last_M = M;
  for (const Task& t : issue) {
    hipStream_t st = p->streams[t.stage];
    const int i = t.stage, m = t.m;
    if (t.kind == 0 && i > 0) rc = hip_ok(hipStreamWaitEvent(st, p->ev_end[p->idx(0, i - 1, m)], 0));
    if (t.kind == 1 && i < S - 1) rc = hip_ok(hipStreamWaitEvent(st, p->ev_end[p->idx(1, i + 1, m)], 0));
    if (rc == STAGE_OK) rc = hip_ok(hipEventRecord(p->ev_start[p->idx(t.kind, i, m)], st));
    if (rc != STAGE_OK) return rc;
    if (t.kind == 0) {
      const void* x = i == 0 ? xs[m] : p->buf(0, i - 1, m);
      void* y = i == S - 1 ? ys[m] : p->buf(0, i, m);
      rc = stage_fwd(p->stages[i], m, x, y, (i == S - 1 && head) ? auxs[m] : nullptr);
    } else {
      const void* dy = i == S - 1 ? (head ? nullptr : dys[m]) : p->buf(1, i, m);
      void* dx = i == 0 ? (emb ? nullptr : dxs[m]) : p->buf(1, i - 1, m);
      rc = stage_bwd(p->stages[i], m, dy, dx);
    }
    if (rc != STAGE_OK) return rc;
    if ((rc = hip_ok(hipEventRecord(p->ev_end[p->idx(t.kind, i, m)], st))) != STAGE_OK) return rc;
  }
  return STAGE_OK;
}

int pipeline_sync(pipeline_handle p) {
  if (!p) return set_error(STAGE_E_NULL, "handle is NULL");
  for (int i = 0; i < p->S; ++i) {
    int rc = stage_sync(p->stages[i]);
    if (rc != STAGE_OK) return rc;
  }
  return STAGE_OK;
}

int pipeline_timeline(pipeline_handle p, double* start_ms, double* end_ms, int capacity) {
  if (!p || !start_ms || !end_ms) return set_error(STAGE_E_NULL, "handle, start_ms and end_ms must not be NULL");
  const int S = p->S, M = p->last_M;
  if (M == 0) return set_error(STAGE_E_BAD_ORDER, "no pipeline_run yet");
  if (capacity < 2 * S * M) return set_error(STAGE_E_BAD_ORDER, "capacity %d too small for %d tasks", capacity, 2 * S * M);
  for (int kind = 0; kind < 2; ++kind)
    for (int i = 0; i < S; ++i)
      for (int m = 0; m < M; ++m) {
        float a = 0.f, b = 0.f;
        if (hipEventElapsedTime(&a, p->ev_t0, p->ev_start[p->idx(kind, i, m)]) != hipSuccess ||
            hipEventElapsedTime(&b, p->ev_t0, p->ev_end[p->idx(kind, i, m)]) != hipSuccess)
          return set_error(STAGE_E_DEVICE, "hipEventElapsedTime failed (call pipeline_sync first)");
        start_ms[((size_t)kind * S + i) * M + m] = a;
        end_ms[((size_t)kind * S + i) * M + m] = b;
      }
  return STAGE_OK;
}

}  // extern "C"
