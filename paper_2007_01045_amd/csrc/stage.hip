// Host side of the stage library: configuration checks, arena layout, the bounded
// activation-slot allocator, the schedule generator / validator / executor, the
// per-task kernel sequences, and the C ABI declared in dapple_stage.h.
//
// Nothing here touches tensor values: every step of a task is one of the kernels
// in gemm.hip, attention.hip, rowops.hip, embed_head.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/dapple_stage.h"
#include "kernels.h"

using namespace dapple;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

// a library-owned lane next to the caller's stream: on the same compute units when the caller's stream is one of
// the partitions of pipeline_partition_stream_create, an ordinary non-blocking stream otherwise
hipError_t make_lane(hipStream_t like, hipStream_t* out) {
  int n = 0;
  const uint32_t* mask = partition_mask_of(like, &n);
  if (mask) return hipExtStreamCreateWithCUMask(out, (uint32_t)n, mask);
  return hipStreamCreateWithFlags(out, hipStreamNonBlocking);
}

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

enum KClass {
  KC_GEMM_FWD = 0, KC_GEMM_DGRAD, KC_GEMM_WGRAD, KC_ATTN_FWD, KC_ATTN_BWD, KC_LN_FWD, KC_LN_BWD,
  KC_REDUCE, KC_COPY, KC_EMBED, KC_HEAD, KC_COUNT
};
const char* const kClassNames[KC_COUNT] = {"gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "ln_fwd",
                                           "ln_bwd",   "reduce",     "copy_zero",  "embed",    "head"};

// element offsets of one layer's tensors in the flat parameter vector
struct LayerParams {
  size_t Wq, bq, Wk, bk, Wv, bv, Wo, bo, ln1g, ln1b, W1, b1, W2, b2, ln2g, ln2b;
};
// byte offsets of one layer's stash inside an activation slot
struct LayerStash {
  size_t qkv, lse, ctx, ctx32, z1, st1, y1, gp, g, z2, st2, y;
};

struct Layout {
  // parameters
  size_t n_params = 0;
  size_t embEw = 0, embEp = 0, embG = 0, embB = 0;
  std::vector<LayerParams> lp;
  size_t hWt = 0, hbt = 0, hG = 0, hB = 0, hEout = 0, hbout = 0;
  // slot
  size_t slot_x0 = 0, slot_ids = 0, slot_embsum = 0, slot_embst = 0;
  std::vector<LayerStash> ls;
  // masked-LM head: NP gathered rows (multiple of 64), VP padded vocabulary (multiple of 64)
  int NP = 0, VP = 0;
  size_t sh_rows = 0, sh_tgt = 0, sh_r = 0, sh_gl = 0, sh_glp = 0, sh_st = 0, sh_t = 0, sh_dz = 0;
  size_t wh_logits = 0, wh_rowloss = 0, wh_dt = 0, wh_dgl = 0, wh_dh = 0, wh_dr = 0, wh_dyfull = 0, wh_part = 0,
         wh_part_cz = 0, wh_info = 0;
  size_t wh_logits2 = 0, wh_rowloss2 = 0, wh_info2 = 0;  // second set: the forward re-run inside a backward task
  size_t we_dx0 = 0, we_de = 0, we_part = 0;
  // fp32 copies of LayerNorm outputs for the residual adds (bf16 stages); set 1: the forward re-run
  // inside a backward task (re-computation), which may overlap a forward task
  size_t ws_y1f[2] = {0, 0}, ws_yf[2][2] = {{0, 0}, {0, 0}};
  size_t slot_bytes = 0;
  // re-computation: a resident micro-batch keeps only its input (and targets); the activations of
  // the task being run live in a buffer of act_bytes: one for forward tasks (arena_fwd_act) and one
  // per backward lane (ws_act, inside each copy of the workspace)
  bool recompute = false;
  int ws_copies = 1;
  size_t act_bytes = 0, st_x = 0, st_aux = 0, ws_act = 0, ws_ydummy = 0, arena_fwd_act = 0;
  // workspace (bytes)
  // buffers the side stream reads exist twice (layers alternate between the sets)
  size_t ws_dx[2] = {0, 0}, ws_dy1 = 0, ws_dctx = 0, ws_delta = 0, ws_head = 0;
  // what the side stream reads of a layer's backward (one set per layer: the backward chain of a task never
  // waits for the side stream before its end)
  struct SideSet { size_t dz2, du, dz1, dqkv, part_ln2, part_ln1; };
  std::vector<SideSet> ws_side;
  size_t workspace_bytes = 0;
  // arena
  size_t grad_bytes = 0, arena_grads = 0, arena_slots = 0, arena_ws = 0, arena_bytes = 0;
};

int check_config(const stage_config& c) {
  if (c.n_layers < 1 || c.hidden < 1 || c.n_heads < 1 || c.ffn < 1 || c.seq < 1 || c.micro_batch < 1)
    return fail(STAGE_E_CONFIG, "n_layers, hidden, n_heads, ffn, seq, micro_batch must be positive");
  if (c.hidden % c.n_heads) return fail(STAGE_E_CONFIG, "hidden (%d) is not a multiple of n_heads (%d)", c.hidden, c.n_heads);
  if (c.max_slots < 1) return fail(STAGE_E_CONFIG, "max_slots must be at least 1");
  if (c.dtype != STAGE_DTYPE_F32 && c.dtype != STAGE_DTYPE_BF16) return fail(STAGE_E_CONFIG, "unknown dtype %d", c.dtype);
  int vec = c.dtype == STAGE_DTYPE_BF16 ? 8 : 4;
  if (c.hidden % vec || c.ffn % vec)
    return fail(STAGE_E_CONFIG, "hidden and ffn must be multiples of %d for this dtype", vec);
  if (c.hidden > 64 * vec * 4) return fail(STAGE_E_CONFIG, "hidden larger than %d is not supported", 64 * vec * 4);
  if (!(c.ln_eps >= 0.f)) return fail(STAGE_E_CONFIG, "ln_eps must be non-negative");
  if (c.has_embedding && c.has_mlm_head)
    return fail(STAGE_E_CONFIG, "a stage has the embedding block or the MLM head, not both");
  if (c.has_embedding || c.has_mlm_head) {
    if (c.vocab < 1) return fail(STAGE_E_CONFIG, "vocab must be positive");
    if (c.has_embedding && c.max_pos < c.seq) return fail(STAGE_E_CONFIG, "max_pos (%d) smaller than seq (%d)", c.max_pos, c.seq);
    if (((long)c.micro_batch * c.seq) % 4) return fail(STAGE_E_CONFIG, "micro_batch * seq must be a multiple of 4 for this stage kind");
    if (c.mlm_max_rows < 0) return fail(STAGE_E_CONFIG, "mlm_max_rows must not be negative");
  }
  if ((long)c.micro_batch * c.seq > (1 << 24)) return fail(STAGE_E_CONFIG, "micro_batch * seq too large");
  return STAGE_OK;
}

void build_layout(const stage_config& c, Layout& L) {
  const size_t H = c.hidden, F = c.ffn, T = (size_t)c.micro_batch * c.seq, E = c.dtype == STAGE_DTYPE_BF16 ? 2 : 4;
  const size_t V = c.vocab, P = c.max_pos;
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += n; return o; };
  if (c.has_embedding) {
    L.embEw = take(V * H); L.embEp = take(P * H); L.embG = take(H); L.embB = take(H);
  }
  L.lp.resize(c.n_layers);
  for (auto& p : L.lp) {
    p.Wq = take(H * H); p.bq = take(H); p.Wk = take(H * H); p.bk = take(H); p.Wv = take(H * H); p.bv = take(H);
    p.Wo = take(H * H); p.bo = take(H); p.ln1g = take(H); p.ln1b = take(H);
    p.W1 = take(H * F); p.b1 = take(F); p.W2 = take(F * H); p.b2 = take(H); p.ln2g = take(H); p.ln2b = take(H);
  }
  if (c.has_mlm_head) {
    L.hWt = take(H * H); L.hbt = take(H); L.hG = take(H); L.hB = take(H); L.hEout = take(V * H); L.hbout = take(V);
  }
  L.n_params = off;

  // activation slot: what F_m leaves for B_m
  size_t so = 0;
  auto stake = [&](size_t bytes) { size_t o = so; so += align_up(bytes); return o; };
  const size_t U = T * H * E;
  if (c.has_embedding) {
    L.slot_ids = stake(T * 4); L.slot_embsum = stake(U); L.slot_embst = stake(2 * T * 4);
  }
  L.slot_x0 = stake(U);
  L.ls.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    auto& s = L.ls[l];
    s.qkv = stake(3 * U);   // q, k, v contiguous (3U is a multiple of 256 whenever U is)
    s.lse = stake((size_t)c.micro_batch * c.n_heads * c.seq * 4);
    // z1, z2 (the pre-LayerNorm sums = the residual stream) are fp32 whatever the stage dtype
    s.ctx = stake(U); s.ctx32 = c.dtype == STAGE_DTYPE_BF16 ? stake(T * H * 4) : 0; s.z1 = stake(T * H * 4); s.st1 = stake(2 * T * 4); s.y1 = stake(U);
    s.gp = stake(T * F * E); s.g = stake(T * F * E); s.z2 = stake(T * H * 4); s.st2 = stake(2 * T * 4);
    bool keep_y = l + 1 < c.n_layers || c.has_mlm_head;
    s.y = keep_y ? stake(U) : 0;
  }
  if (c.has_mlm_head) {
    int cap = c.mlm_max_rows > 0 && c.mlm_max_rows < (int)T ? c.mlm_max_rows : (int)T;
    L.NP = (cap + 63) / 64 * 64;
    L.VP = (c.vocab + 63) / 64 * 64;
    const size_t NP = L.NP, VP = L.VP;
    L.sh_rows = stake(NP * 4); L.sh_tgt = stake(NP * 4); L.sh_r = stake(NP * H * E); L.sh_gl = stake(NP * H * E);
    L.sh_glp = stake(NP * H * E); L.sh_st = stake(2 * NP * 4); L.sh_t = stake(NP * H * E); L.sh_dz = stake(NP * VP * E);
  }
  L.act_bytes = so;
  L.recompute = (c.flags & STAGE_FLAG_RECOMPUTE) != 0;
  if (L.recompute) {
    size_t st = 0;
    L.st_x = st; st += align_up(c.has_embedding ? T * 4 : U);
    L.st_aux = st; st += c.has_mlm_head ? align_up(T * 4) : 0;
    L.slot_bytes = st;
  } else {
    L.slot_bytes = so;
  }

  size_t wo = 0;
  auto wtake = [&](size_t bytes) { size_t o = wo; wo += align_up(bytes); return o; };
  L.ws_dx[0] = wtake(U); L.ws_dx[1] = wtake(U); L.ws_dy1 = wtake(U); L.ws_dctx = wtake(U);
  // delta of the attention backward: [b, A, s], or one row sum per block of 32 columns, [ceil(H/32)][T]
  L.ws_delta = wtake(std::max((size_t)c.micro_batch * c.n_heads * c.seq, (size_t)((c.hidden + 31) / 32) * T) * 4);
  if (c.dtype == STAGE_DTYPE_BF16) {
    for (int fs = 0; fs < (L.recompute ? 2 : 1); ++fs) {
      L.ws_y1f[fs] = wtake(T * H * 4); L.ws_yf[fs][0] = wtake(T * H * 4); L.ws_yf[fs][1] = wtake(T * H * 4);
    }
  }
  const size_t ln_part = ((T + 7) / 8) * 3 * H * 4;
  L.ws_side.resize(c.n_layers);
  for (auto& ss : L.ws_side) {
    ss.dz2 = wtake(U); ss.du = wtake(T * F * E); ss.dz1 = wtake(U); ss.dqkv = wtake(3 * U);
    ss.part_ln2 = wtake(ln_part); ss.part_ln1 = wtake(ln_part);
  }
  if (c.has_mlm_head) {
    const size_t NP = L.NP, VP = L.VP;
    L.wh_logits = wtake(NP * VP * 4); L.wh_rowloss = wtake(NP * 4); L.wh_dt = wtake(NP * H * E);
    L.wh_dgl = wtake(NP * H * E); L.wh_dh = wtake(NP * H * E); L.wh_dr = wtake(NP * H * E); L.wh_dyfull = wtake(U);
    size_t lp = ((NP + 7) / 8) * 3 * H * 4, cp = ((NP + 63) / 64) * VP * 4;
    // three partial-sum buffers: the LayerNorm backward writes its own on the backward stream while the side
    // stream is still reducing a column sum
    L.wh_part = wtake(lp); L.wh_part_cz = wtake(cp); L.wh_info = wtake(16);
    if (L.recompute) { L.wh_logits2 = wtake(NP * VP * 4); L.wh_rowloss2 = wtake(NP * 4); L.wh_info2 = wtake(16); }
  }
  if (c.has_embedding) {
    L.we_dx0 = wtake(U); L.we_de = wtake(U); L.we_part = wtake(ln_part);
  }
  if (L.recompute) {
    L.ws_act = wtake(L.act_bytes); L.ws_ydummy = wtake(U);
  }
  L.workspace_bytes = wo;

  L.grad_bytes = align_up(L.n_params * 4);
  L.arena_grads = 0;
  L.arena_slots = L.grad_bytes;
  L.arena_fwd_act = L.arena_slots + (size_t)c.max_slots * L.slot_bytes;
  L.arena_ws = L.arena_fwd_act + (L.recompute ? align_up(L.act_bytes) : 0);
  // two copies of the workspace: consecutive backward tasks run on two lanes and must not share
  // temporaries (a stage without lanes has one backward lane and one copy)
  L.ws_copies = (c.flags & STAGE_FLAG_ONE_STREAM) ? 1 : 2;
  L.arena_bytes = L.arena_ws + L.ws_copies * L.workspace_bytes;
}

struct ProfEvent { hipEvent_t a, b; int cls; double flops; int lane; int M, N, K, batch; };

}  // namespace

struct dapple_stage {
  stage_config cfg;
  Layout L;
  Dtype dt;
  bool dry;
  const char* W;   // parameters (device, caller-owned)
  char* arena;
  float* grads;
  hipStream_t st;         // the caller's stream: the critical path (forward; backward data gradients)
  // library-owned: weight / bias / LayerNorm gradient work of every backward task, in task order
  hipStream_t side = nullptr;
  hipStream_t fwd = nullptr;   // library-owned: forward tasks inside stage_run_schedule
  hipStream_t bwd2 = nullptr;  // library-owned: every second backward task inside stage_run_schedule
  hipEvent_t ev_b2done = nullptr;
  hipGraph_t graph = nullptr;          // a captured iteration (stage_graph_capture)
  hipGraphExec_t graph_exec = nullptr;
  uint64_t graph_fwd = 0, graph_bwd = 0, graph_launches = 0;
  int graph_peak = 0;
  bool capturing = false;              // inside stage_graph_capture
  bool ran_eagerly = false;            // kernels' attributes are set on their first eager launch
  hipStream_t cur = nullptr;   // where the task being enqueued puts its main-line kernels (st or fwd)
  std::vector<hipEvent_t> ev_f, ev_b;  // per slot: forward done (fwd lane), backward done (caller's stream)
  hipEvent_t ev_start = nullptr;
  bool serial = false, no_side = false;
  std::vector<hipEvent_t> ev;  // per layer: 4 "inputs ready" events (main -> side) + 1 "layer done" (side -> main)
  std::vector<int> slot_of_mb;   // slot -> micro-batch id, -1 = free
  int live = 0, peak_live = 0;
  uint64_t fwd_tasks = 0, bwd_tasks = 0, launches = 0;
  bool profiling = false;
  std::vector<ProfEvent> events;
  size_t events_used = 0;

  size_t E() const { return cfg.dtype == STAGE_DTYPE_BF16 ? 2 : 4; }
  const char* w(size_t elem_off) const { return W + elem_off * E(); }
  float* gr(size_t elem_off) const { return grads + elem_off; }
  char* slot(int s) const { return arena + L.arena_slots + (size_t)s * L.slot_bytes; }
  size_t ws_shift = 0;  // selects the workspace copy of the task being enqueued
  char* ws(size_t off) const { return arena + L.arena_ws + ws_shift + off; }

  // run one launcher; with profiling on, bracket it with two events
  template <typename Fn>
  int run(int cls, double flops, Fn&& fn) { return run_on(cur, cls, flops, fn); }

  // main -> side: the side stream may start once the main stream has passed this point
  int fork(int layer, int which) {
    if (dry) return STAGE_OK;
    hipEvent_t e = ev[layer * 5 + which];
    if (hipEventRecord(e, cur) != hipSuccess || hipStreamWaitEvent(side, e, 0) != hipSuccess)
      return fail(STAGE_E_DEVICE, "event record / wait failed");
    return STAGE_OK;
  }
  // side -> main, in two halves: mark the side work of a layer done; later make main wait for it
  int side_done(int layer) {
    if (dry) return STAGE_OK;
    if (hipEventRecord(ev[layer * 5 + 4], side) != hipSuccess) return fail(STAGE_E_DEVICE, "event record failed");
    return STAGE_OK;
  }
  int join(int layer) {
    if (dry) return STAGE_OK;
    if (hipStreamWaitEvent(cur, ev[layer * 5 + 4], 0) != hipSuccess) return fail(STAGE_E_DEVICE, "event wait failed");
    return STAGE_OK;
  }

  template <typename Fn>
  int run_on(hipStream_t stream, int cls, double flops, Fn&& fn, const GemmArgs* shape = nullptr) {
    if (dry) { ++launches; return STAGE_OK; }
    ProfEvent* pe = nullptr;
    if (profiling) {
      if (events_used == events.size()) {
        ProfEvent e{};
        if (hipEventCreate(&e.a) != hipSuccess || hipEventCreate(&e.b) != hipSuccess)
          return fail(STAGE_E_DEVICE, "hipEventCreate failed");
        events.push_back(e);
      }
      pe = &events[events_used++];
      pe->cls = cls; pe->flops = flops; pe->lane = stream == st ? 0 : (stream == side ? 1 : (stream == fwd ? 2 : (stream == bwd2 ? 3 : 4)));
      pe->M = shape ? shape->M : 0; pe->N = shape ? shape->N : 0; pe->K = shape ? shape->K : 0; pe->batch = shape ? shape->batch : 0;
      (void)hipEventRecord(pe->a, stream);
    }
    hipError_t e = fn(stream);
    if (pe) (void)hipEventRecord(pe->b, stream);
    ++launches;
    if (e != hipSuccess) return fail(STAGE_E_DEVICE, "kernel launch failed: %s", hipGetErrorString(e));
    return STAGE_OK;
  }

  int gemm(int cls, GemmArgs g, bool on_side = false) {
    if (g.kseg_len == 0) g.kseg_len = g.K;
    if (g.k_valid == 0) g.k_valid = g.K;
    if (g.m_valid == 0) g.m_valid = g.M;
    if (g.n_valid == 0) g.n_valid = g.N;
    if (g.batch == 0) g.batch = 1;
    double flops = 2.0 * g.M * g.N * (double)g.K * g.batch;
    hipStream_t s_ = on_side ? side : cur;
    return run_on(s_, cls, flops, [&](hipStream_t s) { return launch_gemm(dt, g, s); }, &g);
  }

  // sl: where the task's activations live; fs: forward workspace set
  int forward(char* sl, int fs, const void* x, void* y, const void* aux);
  int backward(char* sl, const void* dy, void* dx);
};

#define TRY(expr) do { int rc_ = (expr); if (rc_ != STAGE_OK) return rc_; } while (0)

int dapple_stage::forward(char* sl, int fs, const void* x, void* y, const void* aux) {
  const int H = cfg.hidden, F = cfg.ffn, T = cfg.micro_batch * cfg.seq;
  const size_t U = (size_t)T * H * E();
  (void)aux;
  const char* xin = sl + L.slot_x0;
  // bf16 stages keep the residual stream unrounded: the pre-LayerNorm sums z1, z2 and the copy
  // of each LayerNorm output that feeds the next residual add are fp32; only GEMM operands are bf16
  const bool mixed = dt == DT_BF16;
  const void* resid = xin;            // residual input of the next attention block
  bool resid_f32 = false;
  if (cfg.has_embedding) {
    resid = mixed ? (const void*)ws(L.ws_yf[fs][1]) : (const void*)xin;
    resid_f32 = mixed;
    // x = LN(E_w[id] + E_p[pos]); the ids and the pre-LN sum are kept for the backward
    int32_t* ids = (int32_t*)(sl + L.slot_ids);
    char* esum = sl + L.slot_embsum;
    TRY(run(KC_COPY, 0, [&](hipStream_t q) { return launch_copy(ids, x, (size_t)T * 4, q); }));
    TRY(run(KC_EMBED, 0, [&](hipStream_t q) {
      return launch_embed_gather(dt, ids, w(L.embEw), w(L.embEp), esum, T, cfg.seq, H, cfg.vocab, q);
    }));
    TRY(run(KC_LN_FWD, 0, [&](hipStream_t q) {
      return launch_ln_fwd(dt, esum, false, w(L.embG), w(L.embB), sl + L.slot_x0, mixed ? (float*)ws(L.ws_yf[fs][1]) : nullptr,
                           (float*)(sl + L.slot_embst), T, H, cfg.ln_eps, q);
    }));
  } else {
    TRY(run(KC_COPY, 0, [&](hipStream_t q) { return launch_copy(sl + L.slot_x0, x, U, q); }));
  }
  for (int l = 0; l < cfg.n_layers; ++l) {
    const LayerParams& p = L.lp[l];
    const LayerStash& a = L.ls[l];
    char *qkv = sl + a.qkv, *ctx = sl + a.ctx, *z1 = sl + a.z1, *y1 = sl + a.y1, *gp = sl + a.gp, *g = sl + a.g,
         *z2 = sl + a.z2;
    float *lse = (float*)(sl + a.lse), *st1 = (float*)(sl + a.st1), *st2 = (float*)(sl + a.st2);
    char* yout = (l + 1 < cfg.n_layers || cfg.has_mlm_head) ? sl + a.y : (char*)y;
    {  // q, k, v = x Wq + bq, x Wk + bk, x Wv + bv  (three products in one launch)
      GemmArgs ga{};
      ga.A = xin; ga.lda = H; ga.B = w(p.Wq); ga.ldb = H; ga.b_kstrided = 1; ga.bias = w(p.bq);
      ga.C = qkv; ga.ldc = H; ga.M = T; ga.N = H; ga.K = H; ga.batch = 3;
      ga.sA = 0; ga.sB = (long)H * H + H; ga.sBias = (long)H * H + H; ga.sC = (long)T * H; ga.epi = EPI_BIAS;
      TRY(gemm(KC_GEMM_FWD, ga));
    }
    {
      AttnArgs aa{};
      aa.q = qkv; aa.k = qkv + U; aa.v = qkv + 2 * U; aa.ctx = ctx; aa.lse = lse;
      aa.ctx32 = dt == DT_BF16 ? (float*)(sl + a.ctx32) : nullptr;
      aa.b = cfg.micro_batch; aa.s = cfg.seq; aa.A = cfg.n_heads; aa.d = H / cfg.n_heads; aa.H = H;
      double fl = 4.0 * T * (double)cfg.seq * H;
      TRY(run(KC_ATTN_FWD, fl, [&](hipStream_t q) { return launch_attn_fwd(dt, aa, q); }));
    }
    {  // z1 = x + ctx Wo + bo
      GemmArgs ga{};
      ga.A = ctx; ga.lda = H; ga.B = w(p.Wo); ga.ldb = H; ga.b_kstrided = 1; ga.bias = w(p.bo);
      ga.aux = resid; ga.ldaux = H; ga.C = z1; ga.ldc = H; ga.M = T; ga.N = H; ga.K = H;
      ga.epi = EPI_BIAS | EPI_ADD | (mixed ? EPI_OUT32 : 0) | (resid_f32 ? EPI_AUX32 : 0);
      TRY(gemm(KC_GEMM_FWD, ga));
    }
    float* y1f = mixed ? (float*)ws(L.ws_y1f[fs]) : nullptr;
    TRY(run(KC_LN_FWD, 0, [&](hipStream_t q) {
      return launch_ln_fwd(dt, z1, mixed, w(p.ln1g), w(p.ln1b), y1, y1f, st1, T, H, cfg.ln_eps, q);
    }));
    {  // g = GELU(y1 W1 + b1), gp = GELU'(y1 W1 + b1)
      GemmArgs ga{};
      ga.A = y1; ga.lda = H; ga.B = w(p.W1); ga.ldb = F; ga.b_kstrided = 1; ga.bias = w(p.b1);
      ga.C = g; ga.C2 = gp; ga.ldc = F; ga.M = T; ga.N = F; ga.K = H; ga.epi = EPI_BIAS | EPI_GELU;
      TRY(gemm(KC_GEMM_FWD, ga));
    }
    {  // z2 = y1 + g W2 + b2
      GemmArgs ga{};
      ga.A = g; ga.lda = F; ga.B = w(p.W2); ga.ldb = H; ga.b_kstrided = 1; ga.bias = w(p.b2);
      ga.aux = mixed ? (const void*)y1f : (const void*)y1; ga.ldaux = H; ga.C = z2; ga.ldc = H; ga.M = T; ga.N = H;
      ga.K = F; ga.epi = EPI_BIAS | EPI_ADD | (mixed ? EPI_OUT32 | EPI_AUX32 : 0);
      TRY(gemm(KC_GEMM_FWD, ga));
    }
    float* yf = (mixed && l + 1 < cfg.n_layers) ? (float*)ws(L.ws_yf[fs][l & 1]) : nullptr;
    TRY(run(KC_LN_FWD, 0, [&](hipStream_t q) {
      return launch_ln_fwd(dt, z2, mixed, w(p.ln2g), w(p.ln2b), yout, yf, st2, T, H, cfg.ln_eps, q);
    }));
    xin = yout;
    resid = yf ? (const void*)yf : (const void*)yout;
    resid_f32 = yf != nullptr;
  }
  if (cfg.has_mlm_head) {
    // gather the predicted rows, t = LN(GELU(r Wt + bt)), z = t E_out^T (+ b_out inside the
    // cross-entropy kernel), loss -> y[0]; dz is kept in the slot for the backward
    const int NP = L.NP, VP = L.VP, V = cfg.vocab;
    int32_t *rows_idx = (int32_t*)(sl + L.sh_rows), *tgt = (int32_t*)(sl + L.sh_tgt), *info = (int32_t*)ws(fs ? L.wh_info2 : L.wh_info);
    char *r = sl + L.sh_r, *gl = sl + L.sh_gl, *glp = sl + L.sh_glp, *t = sl + L.sh_t, *dz = sl + L.sh_dz;
    float *hst = (float*)(sl + L.sh_st), *logits = (float*)ws(fs ? L.wh_logits2 : L.wh_logits), *rowloss = (float*)ws(fs ? L.wh_rowloss2 : L.wh_rowloss);
    const int cap = cfg.mlm_max_rows > 0 && cfg.mlm_max_rows < T ? cfg.mlm_max_rows : T;
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) { return launch_mlm_compact((const int32_t*)aux, T, cap, NP, V, rows_idx, tgt, info, q); }));
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) { return launch_gather_rows(dt, xin, rows_idx, r, NP, H, T, q); }));
    {
      GemmArgs ga{};
      ga.A = r; ga.lda = H; ga.B = w(L.hWt); ga.ldb = H; ga.b_kstrided = 1; ga.bias = w(L.hbt);
      ga.C = gl; ga.C2 = glp; ga.ldc = H; ga.M = NP; ga.N = H; ga.K = H; ga.epi = EPI_BIAS | EPI_GELU;
      TRY(gemm(KC_HEAD, ga));
    }
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) { return launch_ln_fwd(dt, gl, false, w(L.hG), w(L.hB), t, nullptr, hst, NP, H, cfg.ln_eps, q); }));
    {
      GemmArgs ga{};
      ga.A = t; ga.lda = H; ga.B = w(L.hEout); ga.ldb = H; ga.n_valid = V;
      ga.C = logits; ga.ldc = VP; ga.M = NP; ga.N = VP; ga.K = H; ga.epi = EPI_OUT32;
      TRY(gemm(KC_HEAD, ga));
    }
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) {
      return launch_mlm_ce(dt, logits, w(L.hbout), rows_idx, tgt, NP, V, VP, cfg.loss_scale, dz, rowloss, (float*)y, q);
    }));
  }
  return STAGE_OK;
}

int dapple_stage::backward(char* sl, const void* dy, void* dx) {
  // Two streams.  The caller's stream runs the chain that produces dx (LayerNorm backward,
  // data-gradient products, attention backward): it is the critical path.  Everything that only
  // feeds the gradient accumulators (weight-gradient products, bias column sums, LayerNorm
  // parameter sums) goes to the side stream as soon as its inputs exist, so those kernels fill
  // the CUs the small data-gradient products leave idle.  All accumulator updates happen on the
  // side stream in program order: the result does not depend on how the two streams interleave.
  const int H = cfg.hidden, F = cfg.ffn, T = cfg.micro_batch * cfg.seq;
  const size_t U = (size_t)T * H * E();
  char *dy1 = ws(L.ws_dy1), *dctx = ws(L.ws_dctx);
  float* delta = (float*)ws(L.ws_delta);
  const char* dyin = (const char*)dy;
  if (cfg.has_mlm_head) {
    // backward of the head: dE_out, db_out, dt -> LN -> GELU gate -> dWt, dbt, dr, scattered back
    // into a full [T,H] gradient of the encoder output (zero on rows that are not predicted)
    const int NP = L.NP, VP = L.VP, V = cfg.vocab;
    int32_t* rows_idx = (int32_t*)(sl + L.sh_rows);
    char *r = sl + L.sh_r, *gl = sl + L.sh_gl, *glp = sl + L.sh_glp, *t = sl + L.sh_t, *dz = sl + L.sh_dz;
    float *hst = (float*)(sl + L.sh_st), *part = (float*)ws(L.wh_part);
    char *dtb = ws(L.wh_dt), *dgl = ws(L.wh_dgl), *dh = ws(L.wh_dh), *dr = ws(L.wh_dr), *dyfull = ws(L.wh_dyfull);
    int nblk = 0;
    // The head's accumulator updates go to the side stream like the layers' (fork events of the pseudo-layer
    // n_layers), in the order dE_out, db_out, LayerNorm gain and shift, dWt, dbt.
    const int HL = cfg.n_layers;
    float* part_cz = (float*)ws(L.wh_part_cz);
    TRY(fork(HL, 0));
    {  // dE_out += dz^T t
      GemmArgs ga{};
      ga.A = dz; ga.lda = VP; ga.a_kstrided = 1; ga.B = t; ga.ldb = H; ga.b_kstrided = 1;
      ga.C = gr(L.hEout); ga.ldc = H; ga.M = V; ga.N = H; ga.K = NP; ga.epi = EPI_ACC32;
      TRY(gemm(KC_HEAD, ga, true));
    }
    TRY(run_on(side, KC_HEAD, 0, [&](hipStream_t q) { return launch_colsum(dt, dz, NP, V, VP, part_cz, gr(L.hbout), 1, 0, 0, q); }));
    {  // dt = dz E_out
      GemmArgs ga{};
      ga.A = dz; ga.lda = VP; ga.B = w(L.hEout); ga.ldb = H; ga.b_kstrided = 1; ga.k_valid = V;
      ga.C = dtb; ga.ldc = H; ga.M = NP; ga.N = H; ga.K = VP;
      TRY(gemm(KC_HEAD, ga));
    }
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) { return launch_ln_bwd(dt, dtb, gl, false, hst, w(L.hG), dgl, part, &nblk, NP, H, q); }));
    TRY(fork(HL, 1));
    TRY(run_on(side, KC_HEAD, 0, [&](hipStream_t q) { return launch_partial_reduce(part, nblk, 3, H, gr(L.hG), gr(L.hB), nullptr, q); }));
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) { return launch_mul(dt, dgl, glp, dh, (long)NP * H, q); }));
    TRY(fork(HL, 0));   // event 0 again: the side stream's first wait on it is already enqueued
    {  // dWt += r^T dh, dbt += the column sums of dh
      GemmArgs ga{};
      ga.A = r; ga.lda = H; ga.a_kstrided = 1; ga.B = dh; ga.ldb = H; ga.b_kstrided = 1;
      ga.C = gr(L.hWt); ga.ldc = H; ga.M = H; ga.N = H; ga.K = NP; ga.epi = EPI_ACC32 | EPI_BSUM;
      ga.bsum_z[0] = gr(L.hbt);
      TRY(gemm(KC_HEAD, ga, true));
    }
    TRY(side_done(HL));
    {  // dr = dh Wt^T
      GemmArgs ga{};
      ga.A = dh; ga.lda = H; ga.B = w(L.hWt); ga.ldb = H; ga.C = dr; ga.ldc = H; ga.M = NP; ga.N = H; ga.K = H;
      TRY(gemm(KC_HEAD, ga));
    }
    TRY(run(KC_COPY, 0, [&](hipStream_t q) { return launch_zero(dyfull, U, q); }));
    TRY(run(KC_HEAD, 0, [&](hipStream_t q) { return launch_scatter_rows(dt, dr, rows_idx, dyfull, NP, H, T, q); }));
    dyin = dyfull;
  }
  for (int l = cfg.n_layers - 1; l >= 0; --l) {
    const LayerParams& p = L.lp[l];
    const LayerStash& a = L.ls[l];
    const Layout::SideSet& ss = L.ws_side[l];  // this layer's buffers that the side stream reads
    char *dz2 = ws(ss.dz2), *du = ws(ss.du), *dz1 = ws(ss.dz1), *dqkv = ws(ss.dqkv);
    float *part_ln2 = (float*)ws(ss.part_ln2), *part_ln1 = (float*)ws(ss.part_ln1);
    const char* xl = l == 0 ? sl + L.slot_x0 : sl + L.ls[l - 1].y;
    char *qkv = sl + a.qkv, *ctx = sl + a.ctx, *z1 = sl + a.z1, *y1 = sl + a.y1, *gp = sl + a.gp, *g = sl + a.g,
         *z2 = sl + a.z2;
    float *lse = (float*)(sl + a.lse), *st1 = (float*)(sl + a.st1), *st2 = (float*)(sl + a.st2);
    char* dxout = l == 0 ? (cfg.has_embedding ? ws(L.we_dx0) : (char*)dx) : ws(L.ws_dx[l & 1]);
    const size_t pstride = (size_t)H * H + H;
    int nblk = 0;

    // y = LN(z2): dz2, and block partial sums for the gradients of ln2 gain/shift and of b2
    TRY(run(KC_LN_BWD, 0, [&](hipStream_t q) { return launch_ln_bwd(dt, dyin, z2, dt == DT_BF16, st2, w(p.ln2g), dz2, part_ln2, &nblk, T, H, q); }));
    // One side stream: the layer's bias and LayerNorm-parameter reductions wait and go out as ONE
    // launch after the last weight-gradient product (the side stream is the longest chain of a
    // step, and a small kernel costs it a dispatch of ~15 us when the GPU is full).  Each
    // reduction adds in the same order as the stand-alone kernels.
    const int nblk_ln2 = nblk;
    {  // du = (dz2 W2^T) o GELU'(u)
      GemmArgs ga{};
      ga.A = dz2; ga.lda = H; ga.B = w(p.W2); ga.ldb = H; ga.aux = gp; ga.ldaux = F;
      ga.C = du; ga.ldc = F; ga.M = T; ga.N = F; ga.K = H; ga.epi = EPI_MUL;
      TRY(gemm(KC_GEMM_DGRAD, ga));
    }
    // two forks per layer (here and after the attention backward), not one per side launch: every event
    // recorded on this stream sits between two kernels of the task's chain (14.17 -> 14.14 ms; a single fork per
    // layer holds the side stream back too long: 14.35)
    TRY(fork(l, 1));
    {  // dW2 += g^T dz2
      GemmArgs ga{};
      ga.A = g; ga.lda = F; ga.a_kstrided = 1; ga.B = dz2; ga.ldb = H; ga.b_kstrided = 1;
      ga.C = gr(p.W2); ga.ldc = H; ga.M = F; ga.N = H; ga.K = T; ga.epi = EPI_ACC32;
      TRY(gemm(KC_GEMM_WGRAD, ga, true));
    }
    {  // dW1 += y1^T du, and db1 += the column sums of du in the same launch
      GemmArgs ga{};
      ga.A = y1; ga.lda = H; ga.a_kstrided = 1; ga.B = du; ga.ldb = F; ga.b_kstrided = 1;
      ga.C = gr(p.W1); ga.ldc = F; ga.M = H; ga.N = F; ga.K = T; ga.epi = EPI_ACC32 | EPI_BSUM;
      ga.bsum_z[0] = gr(p.b1);
      TRY(gemm(KC_GEMM_WGRAD, ga, true));
    }
    {  // dy1 = du W1^T + dz2 (residual branch)
      GemmArgs ga{};
      ga.A = du; ga.lda = F; ga.B = w(p.W1); ga.ldb = F; ga.aux = dz2; ga.ldaux = H;
      ga.C = dy1; ga.ldc = H; ga.M = T; ga.N = H; ga.K = F; ga.epi = EPI_ADD;
      TRY(gemm(KC_GEMM_DGRAD, ga));
    }
    TRY(run(KC_LN_BWD, 0, [&](hipStream_t q) { return launch_ln_bwd(dt, dy1, z1, dt == DT_BF16, st1, w(p.ln1g), dz1, part_ln1, &nblk, T, H, q); }));
    const int nblk_ln1 = nblk;
    AttnArgs aa{};
    aa.q = qkv; aa.k = qkv + U; aa.v = qkv + 2 * U; aa.ctx = ctx; aa.lse = lse; aa.dctx = dctx;
    aa.ctx32 = dt == DT_BF16 ? (float*)(sl + a.ctx32) : nullptr;
    aa.dq = dqkv; aa.dk = dqkv + U; aa.dv = dqkv + 2 * U; aa.delta = delta;
    aa.b = cfg.micro_batch; aa.s = cfg.seq; aa.A = cfg.n_heads; aa.d = H / cfg.n_heads; aa.H = H;
    {  // dctx = dz1 Wo^T; where the MFMA kernels run, its epilogue also leaves rowsum(dctx o ctx) per block of
       // 32 columns, the delta of the attention backward
      GemmArgs ga{};
      ga.A = dz1; ga.lda = H; ga.B = w(p.Wo); ga.ldb = H; ga.C = dctx; ga.ldc = H; ga.M = T; ga.N = H; ga.K = H;
      if (aa.ctx32 && attn_uses_mfma(dt, aa)) {
        GemmArgs probe = ga;
        probe.epi = EPI_ROWDOT | EPI_AUX32; probe.aux = aa.ctx32; probe.ldaux = H; probe.rowdot = delta;
        probe.batch = 1; probe.kseg_len = ga.K; probe.k_valid = ga.K; probe.m_valid = ga.M; probe.n_valid = ga.N;
        if (gemm_uses_mfma(dt, probe)) {
          ga = probe;
          aa.delta_blocks = delta;
        }
      }
      TRY(gemm(KC_GEMM_DGRAD, ga));
    }
    {
      double fl = 8.0 * T * (double)cfg.seq * H;
      TRY(run(KC_ATTN_BWD, fl, [&](hipStream_t q) { return launch_attn_bwd(dt, aa, q); }));
    }
    TRY(fork(l, 3));
    {  // dWq, dWk, dWv += x^T dq, x^T dk, x^T dv and dWo += ctx^T dz1: four products of one
       // shape in one launch (alone, each would leave most of the CUs idle); the first three
       // also add the column sums of dq, dk, dv to the bias gradients
      GemmArgs ga{};
      ga.lda = H; ga.a_kstrided = 1; ga.ldb = H; ga.b_kstrided = 1;
      ga.ldc = H; ga.M = H; ga.N = H; ga.K = T; ga.batch = 4; ga.epi = EPI_ACC32 | EPI_BSUM;
      for (int z = 0; z < 3; ++z) {
        ga.Az[z] = xl; ga.Bz[z] = dqkv + z * U; ga.Cz[z] = gr(p.Wq + z * pstride);
        ga.bsum_z[z] = gr(p.bq + z * pstride);
      }
      ga.Az[3] = ctx; ga.Bz[3] = dz1; ga.Cz[3] = gr(p.Wo);
      ga.A = ga.Az[0]; ga.B = ga.Bz[0]; ga.C = ga.Cz[0];
      TRY(gemm(KC_GEMM_WGRAD, ga, true));
    }
    {
      ReduceJobs J{};
      auto add = [&](const float* partial, long stride, int nb, int cols, float* out) {
        J.j[J.n++] = ReduceJob{partial, out, nb, cols, stride};
      };
      float* o2[3] = {gr(p.ln2g), gr(p.ln2b), gr(p.b2)};
      float* o1[3] = {gr(p.ln1g), gr(p.ln1b), gr(p.bo)};
      for (int v = 0; v < 3; ++v) add(part_ln2 + (size_t)v * H, 3L * H, nblk_ln2, H, o2[v]);
      for (int v = 0; v < 3; ++v) add(part_ln1 + (size_t)v * H, 3L * H, nblk_ln1, H, o1[v]);
      TRY(run_on(side, KC_REDUCE, 0, [&](hipStream_t q) { return launch_reduce_jobs(J, q); }));
    }
    TRY(side_done(l));
    {  // dx = dq Wq^T + dk Wk^T + dv Wv^T + dz1 (residual branch): one product over K = 3H
      GemmArgs ga{};
      ga.A = dqkv; ga.lda = H; ga.B = w(p.Wq); ga.ldb = H; ga.aux = dz1; ga.ldaux = H;
      ga.C = dxout; ga.ldc = H; ga.M = T; ga.N = H; ga.K = 3 * H; ga.kseg_len = H;
      ga.segA = (long)T * H; ga.segB = (long)pstride; ga.epi = EPI_ADD;
      TRY(gemm(KC_GEMM_DGRAD, ga));
    }
    dyin = dxout;
  }
  if (cfg.has_embedding) {
    // x = LN(e): de, the gradients of the embedding LayerNorm, then the two table gradients
    char *de = ws(L.we_de), *esum = sl + L.slot_embsum;
    float* part = (float*)ws(L.we_part);
    int nblk = 0;
    TRY(run(KC_EMBED, 0, [&](hipStream_t q) {
      return launch_ln_bwd(dt, dyin, esum, false, (const float*)(sl + L.slot_embst), w(L.embG), de, part, &nblk, T, H, q);
    }));
    // the three accumulations (LayerNorm gain and shift, the two tables) join the side stream's queue like every
    // other accumulator update, so that backward tasks may run on two lanes: fork event 3 of layer 0 is free
    // again (its side work was enqueued above), and the task's closing join below waits for this too
    TRY(fork(0, 3));
    TRY(run_on(side, KC_EMBED, 0, [&](hipStream_t q) { return launch_partial_reduce(part, nblk, 3, H, gr(L.embG), gr(L.embB), nullptr, q); }));
    TRY(run_on(side, KC_EMBED, 0, [&](hipStream_t q) {
      return launch_embed_bwd(dt, (const int32_t*)(sl + L.slot_ids), de, gr(L.embEw), gr(L.embEp), cfg.micro_batch,
                              cfg.seq, H, cfg.vocab, q);
    }));
    TRY(side_done(0));
  }
  // The task ends when both streams are done: whatever follows on the caller's stream (the next
  // forward reusing this slot, a gradient read-out) is ordered after the accumulator updates.
  // (the side stream is in order and layer 0's work is the last it was given)
  TRY(join(0));
  return STAGE_OK;
}

// ------------------------------------------------------------------ schedule
static int make_schedule(int M, int K, int order, std::vector<int32_t>& ops) {
  if (M < 1 || K < 1) return fail(STAGE_E_BAD_ORDER, "M and K must be positive (M=%d, K=%d)", M, K);
  ops.clear();
  if (order == STAGE_ORDER_GPIPE) {
    for (int m = 0; m < M; ++m) ops.push_back(m + 1);
    for (int m = 0; m < M; ++m) ops.push_back(-(m + 1));
  } else if (order == STAGE_ORDER_EARLY_BACKWARD) {
    int Kp = K < M ? K : M;
    for (int m = 0; m < Kp; ++m) ops.push_back(m + 1);          // warm-up: inject K' micro-batches
    for (int j = 0; j + Kp < M; ++j) {                          // steady: B_j frees what F_{j+K'} reuses
      ops.push_back(-(j + 1));
      ops.push_back(j + Kp + 1);
    }
    for (int m = M - Kp; m < M; ++m) ops.push_back(-(m + 1));   // drain
  } else {
    return fail(STAGE_E_BAD_ORDER, "unknown order %d", order);
  }
  return STAGE_OK;
}

// each micro-batch forward once then backward once, at most `limit` resident
static int validate_ops(const int32_t* ops, int n, int M, int limit) {
  if (n != 2 * M) return fail(STAGE_E_BAD_ORDER, "task list has %d entries, expected %d", n, 2 * M);
  std::vector<int> state(M, 0);
  int live = 0;
  for (int i = 0; i < n; ++i) {
    int m = (ops[i] > 0 ? ops[i] : -ops[i]) - 1;
    if (ops[i] == 0 || m >= M) return fail(STAGE_E_BAD_ORDER, "task %d names micro-batch %d outside [0,%d)", i, m, M);
    if (ops[i] > 0) {
      if (state[m] != 0) return fail(STAGE_E_BAD_ORDER, "task %d: F%d twice", i, m);
      if (live >= limit) return fail(STAGE_E_BAD_ORDER, "task %d: F%d would make %d micro-batches resident (limit %d)", i, m, live + 1, limit);
      state[m] = 1; ++live;
    } else {
      if (state[m] != 1) return fail(STAGE_E_BAD_ORDER, "task %d: B%d without a live F%d", i, m, m);
      state[m] = 2; --live;
    }
  }
  return STAGE_OK;
}

// ------------------------------------------------------------------ C ABI
namespace dapple {
int set_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
}  // namespace dapple

extern "C" {

const char* stage_last_error(void) { return g_err.c_str(); }

int stage_query_sizes(const stage_config* cfg, stage_sizes* out) {
  if (!cfg || !out) return fail(STAGE_E_NULL, "cfg and out must not be NULL");
  TRY(check_config(*cfg));
  Layout L;
  build_layout(*cfg, L);
  out->n_params = L.n_params;
  out->weight_bytes = L.n_params * (cfg->dtype == STAGE_DTYPE_BF16 ? 2 : 4);
  out->grad_bytes = L.grad_bytes;
  out->slot_bytes = L.slot_bytes;
  out->workspace_bytes = L.workspace_bytes;
  out->arena_bytes = L.arena_bytes;
  return STAGE_OK;
}

int stage_init(stage_handle* out, const stage_config* cfg, const void* weights_dev, void* arena_dev,
               size_t arena_bytes, void* hip_stream) {
  if (!out || !cfg) return fail(STAGE_E_NULL, "out and cfg must not be NULL");
  TRY(check_config(*cfg));
  const bool dry = (cfg->flags & STAGE_FLAG_DRY_RUN) != 0;
  if (!dry && (!weights_dev || !arena_dev)) return fail(STAGE_E_NULL, "weights_dev and arena_dev must not be NULL");
  dapple_stage* h = new (std::nothrow) dapple_stage();
  if (!h) return fail(STAGE_E_DEVICE, "out of host memory");
  h->cfg = *cfg;
  build_layout(*cfg, h->L);
  if (!dry) {
    if (arena_bytes < h->L.arena_bytes) {
      size_t need = h->L.arena_bytes;
      delete h;
      return fail(STAGE_E_ARENA_SMALL, "arena has %zu bytes, %zu needed", arena_bytes, need);
    }
    if (((uintptr_t)arena_dev & 255) || ((uintptr_t)weights_dev & 15)) {
      delete h;
      return fail(STAGE_E_CONFIG, "arena_dev must be 256-byte aligned and weights_dev 16-byte aligned");
    }
  }
  h->dt = cfg->dtype == STAGE_DTYPE_BF16 ? DT_BF16 : DT_F32;
  h->dry = dry;
  h->W = (const char*)weights_dev;
  h->arena = (char*)arena_dev;
  h->grads = (float*)arena_dev;
  h->st = (hipStream_t)hip_stream;
  h->slot_of_mb.assign(cfg->max_slots, -1);
  if (!dry) {
    // default priority on purpose; the side stream never outlives the handle
    h->serial = h->no_side = (cfg->flags & STAGE_FLAG_ONE_STREAM) != 0;
    if (h->no_side) {
      h->side = h->st;
    } else {
      hipError_t e = make_lane(h->st, &h->side);
      if (e != hipSuccess) {
        delete h;
        return fail(STAGE_E_DEVICE, "creating the side stream failed: %s", hipGetErrorString(e));
      }
    }
    // the forward lane and the second backward lane are made by the first stage_run_schedule that uses lanes:
    // a stage driven task by task (stage_fwd / stage_bwd, the pipeline of several stages) holds no idle queues
    h->ev.resize((size_t)(cfg->n_layers + 1) * 5);   // one more set for the head's side work
    h->ev_f.resize(cfg->max_slots);
    h->ev_b.resize(cfg->max_slots);
    std::vector<hipEvent_t*> all;
    for (auto& e : h->ev) all.push_back(&e);
    for (auto& e : h->ev_f) all.push_back(&e);
    for (auto& e : h->ev_b) all.push_back(&e);
    all.push_back(&h->ev_start);
    all.push_back(&h->ev_b2done);
    for (hipEvent_t* e : all)
      if (hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess) {
        delete h;
        return fail(STAGE_E_DEVICE, "hipEventCreate failed");
      }
  }
  h->cur = h->st;
  int rc = h->run(KC_COPY, 0, [&](hipStream_t q) { return launch_zero(h->grads, h->L.grad_bytes, q); });
  if (rc == STAGE_OK && cfg->has_mlm_head) {
    rc = h->run(KC_COPY, 0, [&](hipStream_t q) { return launch_zero(h->ws(h->L.wh_info), 16, q); });
    for (int c = 0; rc == STAGE_OK && h->L.recompute && c < h->L.ws_copies; ++c)   // one flag per backward lane
      rc = h->run(KC_COPY, 0, [&](hipStream_t q) {
        return launch_zero(h->ws((size_t)c * h->L.workspace_bytes + h->L.wh_info2), 16, q);
      });
  }
  if (rc != STAGE_OK) { delete h; return rc; }
  *out = h;
  return STAGE_OK;
}

int stage_destroy(stage_handle h) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (!h->dry) {
    (void)hipStreamSynchronize(h->st);
    if (h->side) (void)hipStreamSynchronize(h->side);
    if (h->fwd) (void)hipStreamSynchronize(h->fwd);
    if (h->bwd2) (void)hipStreamSynchronize(h->bwd2);
  }
  if (h->graph_exec) (void)hipGraphExecDestroy(h->graph_exec);
  if (h->graph) (void)hipGraphDestroy(h->graph);
  for (auto& e : h->events) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  for (auto& e : h->ev) (void)hipEventDestroy(e);
  for (auto& e : h->ev_f) (void)hipEventDestroy(e);
  for (auto& e : h->ev_b) (void)hipEventDestroy(e);
  if (h->ev_start) (void)hipEventDestroy(h->ev_start);
  if (h->ev_b2done) (void)hipEventDestroy(h->ev_b2done);
  if (h->bwd2) (void)hipStreamDestroy(h->bwd2);
  if (h->side && h->side != h->st) (void)hipStreamDestroy(h->side);
  if (h->fwd) (void)hipStreamDestroy(h->fwd);
  delete h;
  return STAGE_OK;
}

static int find_slot(stage_handle h, int mb) {
  for (size_t i = 0; i < h->slot_of_mb.size(); ++i)
    if (h->slot_of_mb[i] == mb) return (int)i;
  return -1;
}

int stage_fwd(stage_handle h, int mb, const void* x_dev, void* y_dev, const void* aux_dev) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (mb < 0) return fail(STAGE_E_BAD_ORDER, "micro-batch index %d is negative", mb);
  if (!h->dry && (!x_dev || !y_dev)) return fail(STAGE_E_NULL, "x_dev and y_dev must not be NULL");
  if (!h->dry && h->cfg.has_mlm_head && !aux_dev) return fail(STAGE_E_NULL, "aux_dev (targets) must not be NULL");
  if (find_slot(h, mb) >= 0) return fail(STAGE_E_DUP_MB, "micro-batch %d is already resident", mb);
  int s = find_slot(h, -1);
  if (s < 0) return fail(STAGE_E_NO_SLOT, "all %d activation slots are in use", h->cfg.max_slots);
  if (h->L.recompute && !h->dry) {
    // keep only what the forward cannot be re-run without: the input (token ids on a first stage)
    // and the targets; the activations go to the forward tasks' buffer and are dropped
    char* stash = h->slot(s);
    const Layout& L = h->L;
    const size_t xb = h->cfg.has_embedding ? (size_t)h->cfg.micro_batch * h->cfg.seq * 4
                                            : (size_t)h->cfg.micro_batch * h->cfg.seq * h->cfg.hidden * h->E();
    TRY(h->run(KC_COPY, 0, [&](hipStream_t q) { return launch_copy(stash + L.st_x, x_dev, xb, q); }));
    if (h->cfg.has_mlm_head)
      TRY(h->run(KC_COPY, 0, [&](hipStream_t q) {
        return launch_copy(stash + L.st_aux, aux_dev, (size_t)h->cfg.micro_batch * h->cfg.seq * 4, q);
      }));
    TRY(h->forward(h->arena + L.arena_fwd_act, 0, x_dev, y_dev, aux_dev));
  } else {
    TRY(h->forward(h->slot(s), 0, x_dev, y_dev, aux_dev));
  }
  h->slot_of_mb[s] = mb;
  ++h->live;
  if (h->live > h->peak_live) h->peak_live = h->live;
  ++h->fwd_tasks;
  return STAGE_OK;
}

int stage_bwd(stage_handle h, int mb, const void* dy_dev, void* dx_dev) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (!h->dry && !h->cfg.has_mlm_head && !dy_dev) return fail(STAGE_E_NULL, "dy_dev must not be NULL");
  if (!h->dry && !h->cfg.has_embedding && !dx_dev) return fail(STAGE_E_NULL, "dx_dev must not be NULL");
  int s = mb < 0 ? -1 : find_slot(h, mb);
  if (s < 0) return fail(STAGE_E_NOT_RESIDENT, "micro-batch %d has no live forward", mb);
  if (h->L.recompute && !h->dry) {
    // re-run the forward from the kept input into the backward tasks' buffer, then go backward
    const Layout& L = h->L;
    char *stash = h->slot(s), *act = h->ws(L.ws_act);
    TRY(h->forward(act, 1, stash + L.st_x, h->ws(L.ws_ydummy), h->cfg.has_mlm_head ? stash + L.st_aux : nullptr));
    TRY(h->backward(act, dy_dev, dx_dev));
  } else {
    TRY(h->backward(h->slot(s), dy_dev, dx_dev));
  }
  h->slot_of_mb[s] = -1;   // released after its backward: the next injected micro-batch reuses it
  --h->live;
  ++h->bwd_tasks;
  return STAGE_OK;
}

int stage_schedule_ops(int M, int K, int order, int32_t* ops_out, int capacity) {
  if (!ops_out) return fail(STAGE_E_NULL, "ops_out must not be NULL");
  std::vector<int32_t> ops;
  TRY(make_schedule(M, K, order, ops));
  if ((int)ops.size() > capacity) return fail(STAGE_E_BAD_ORDER, "capacity %d too small for %zu tasks", capacity, ops.size());
  memcpy(ops_out, ops.data(), ops.size() * sizeof(int32_t));
  return (int)ops.size();
}

static int ensure_lanes(stage_handle h) {
  if (h->fwd) return STAGE_OK;
  hipError_t e = make_lane(h->st, &h->fwd);
  if (e == hipSuccess) e = make_lane(h->st, &h->bwd2);
  if (e != hipSuccess) return fail(STAGE_E_DEVICE, "creating the forward / second backward stream failed: %s", hipGetErrorString(e));
  return STAGE_OK;
}

int stage_run_schedule(stage_handle h, int M, int K, int order, const void* const* xs, const void* const* dys,
                       void* const* ys, void* const* dxs, const void* const* auxs, const int32_t* explicit_ops,
                       int n_ops) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (M < 1 || K < 1) return fail(STAGE_E_BAD_ORDER, "M and K must be positive (M=%d, K=%d)", M, K);
  std::vector<int32_t> ops;
  int limit;
  if (order == STAGE_ORDER_EXPLICIT) {
    if (!explicit_ops) return fail(STAGE_E_NULL, "explicit_ops must not be NULL");
    ops.assign(explicit_ops, explicit_ops + (n_ops > 0 ? n_ops : 0));
    limit = K;
  } else {
    TRY(make_schedule(M, K, order, ops));
    limit = order == STAGE_ORDER_GPIPE ? M : (K < M ? K : M);
  }
  if (limit > h->cfg.max_slots)
    return fail(STAGE_E_BAD_ORDER, "this order keeps %d micro-batches resident, the stage has %d slots", limit, h->cfg.max_slots);
  TRY(validate_ops(ops.data(), (int)ops.size(), M, limit));
  if (h->live != 0) return fail(STAGE_E_BAD_ORDER, "%d micro-batches are still resident from earlier calls", h->live);
  if (!h->dry) {
    const bool need_dy = !h->cfg.has_mlm_head, need_dx = !h->cfg.has_embedding, need_aux = h->cfg.has_mlm_head;
    if (!xs || !ys || (need_dy && !dys) || (need_dx && !dxs) || (need_aux && !auxs))
      return fail(STAGE_E_NULL, "a required pointer array is NULL");
    for (int m = 0; m < M; ++m)
      if (!xs[m] || !ys[m] || (need_dy && !dys[m]) || (need_dx && !dxs[m]) || (need_aux && !auxs[m]))
        return fail(STAGE_E_NULL, "a device pointer of micro-batch %d is NULL", m);
  }
  // Two lanes: forward tasks go to the library's forward stream, backward tasks stay on the
  // caller's stream, so that F_{j+K} runs beside B_{j+1} instead of between B_j and B_{j+1}.
  // Dependences kept: F_m -> B_m; B_m -> the forward that reuses its slot; forwards among
  // themselves and backwards among themselves in list order (which fixes the order of every
  // gradient accumulation).  The early-backward order needs no more than that; the other orders
  // are run strictly as listed (a backward waits for every forward listed before it).
  const bool lanes = !h->dry && !h->profiling && !h->serial;
  const bool strict = order != STAGE_ORDER_EARLY_BACKWARD;
  std::vector<char> b_pending(h->cfg.max_slots, 0);
  int last_f_slot = -1;
  auto hip_ok = [](hipError_t e) { return e == hipSuccess ? STAGE_OK : fail(STAGE_E_DEVICE, "%s", hipGetErrorString(e)); };
  // Early-backward order, plain stages: consecutive backward tasks alternate between the caller's
  // stream and a second backward stream (each with its own copy of the workspace), so the head of
  // B_{j+1} overlaps the tail of B_j.  Their accumulator updates still happen in list order: all of
  // them are issued, in host order, on the one side stream (the embedding block's and the head's too).
  // A capture keeps to one backward lane: the HIP runtime that ships with PyTorch 2.10 (ROCm 7.0) recurses
  // without end in hipStreamEndCapture once two streams other than the capture's origin have waited for each
  // other's events (side lane <-> second backward lane); the origin may wait for and be waited for by anyone.
  // (The GPipe order alternates its backward tasks the same way once every forward is done; an explicit list
  // keeps one backward lane.)
  const bool two = lanes && order != STAGE_ORDER_EXPLICIT && h->L.ws_copies == 2 &&
                   !h->no_side && !h->capturing;
  int n_bwd = 0;
  bool used_b2 = false;
  if (lanes) TRY(ensure_lanes(h));
  if (lanes) {
    TRY(hip_ok(hipEventRecord(h->ev_start, h->st)));
    TRY(hip_ok(hipStreamWaitEvent(h->fwd, h->ev_start, 0)));
  }
  int rc = STAGE_OK;
  for (int32_t op : ops) {
    int m = (op > 0 ? op : -op) - 1;
    if (op > 0) {
      if (lanes) {
        int s = find_slot(h, -1);  // the slot stage_fwd is about to take
        if (s >= 0 && b_pending[s]) {
          if ((rc = hip_ok(hipStreamWaitEvent(h->fwd, h->ev_b[s], 0))) != STAGE_OK) break;
          b_pending[s] = 0;
        }
        h->cur = h->fwd;
        rc = stage_fwd(h, m, xs[m], ys[m], auxs ? auxs[m] : nullptr);
        h->cur = h->st;
        if (rc != STAGE_OK) break;
        if ((rc = hip_ok(hipEventRecord(h->ev_f[s], h->fwd))) != STAGE_OK) break;
        last_f_slot = s;
      } else if ((rc = stage_fwd(h, m, xs ? xs[m] : nullptr, ys ? ys[m] : nullptr, auxs ? auxs[m] : nullptr)) != STAGE_OK) break;
    } else {
      int s = -1;
      const bool second = two && (n_bwd & 1);
      hipStream_t bs = second ? h->bwd2 : h->st;
      ++n_bwd;
      if (lanes) {
        if (second && !used_b2) {
          if ((rc = hip_ok(hipStreamWaitEvent(bs, h->ev_start, 0))) != STAGE_OK) break;
          used_b2 = true;
        }
        s = find_slot(h, m);
        int w = strict ? last_f_slot : s;
        if (w >= 0 && (rc = hip_ok(hipStreamWaitEvent(bs, h->ev_f[w], 0))) != STAGE_OK) break;
      }
      h->cur = bs;
      h->ws_shift = second ? h->L.workspace_bytes : 0;
      rc = stage_bwd(h, m, dys ? dys[m] : nullptr, dxs ? dxs[m] : nullptr);
      h->cur = h->st;
      h->ws_shift = 0;
      if (rc != STAGE_OK) break;
      if (lanes) {
        if ((rc = hip_ok(hipEventRecord(h->ev_b[s], bs))) != STAGE_OK) break;
        b_pending[s] = 1;
      }
    }
  }
  // the caller's stream ends behind everything the forward lane was given, also on an error
  if (lanes && last_f_slot >= 0) {
    int rc2 = hip_ok(hipStreamWaitEvent(h->st, h->ev_f[last_f_slot], 0));
    if (rc == STAGE_OK) rc = rc2;
  }
  if (used_b2) {  // ... and behind the second backward lane
    int rc2 = hip_ok(hipEventRecord(h->ev_b2done, h->bwd2));
    if (rc2 == STAGE_OK) rc2 = hip_ok(hipStreamWaitEvent(h->st, h->ev_b2done, 0));
    if (rc == STAGE_OK) rc = rc2;
  }
  if (rc == STAGE_OK && !h->dry) h->ran_eagerly = true;
  return rc;
}

int stage_graph_capture(stage_handle h, int M, int K, int order, const void* const* xs, const void* const* dys,
                        void* const* ys, void* const* dxs, const void* const* auxs, const int32_t* explicit_ops,
                        int n_ops, int zero_grads_first) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (h->dry) return fail(STAGE_E_CONFIG, "a dry-run stage launches nothing to capture");
  if (!h->st) return fail(STAGE_E_CONFIG, "the stage was created on the default (NULL) stream, which cannot be captured");
  if (h->profiling) return fail(STAGE_E_CONFIG, "switch per-launch timing off before capturing");
  if (!h->ran_eagerly)
    return fail(STAGE_E_BAD_ORDER, "run the same iteration once with stage_run_schedule before capturing it");
  if (h->live != 0) return fail(STAGE_E_BAD_ORDER, "%d micro-batches are still resident", h->live);
  if (h->graph_exec) { (void)hipGraphExecDestroy(h->graph_exec); h->graph_exec = nullptr; }
  if (h->graph) { (void)hipGraphDestroy(h->graph); h->graph = nullptr; }
  if (!h->serial) TRY(ensure_lanes(h));   // no stream is created inside a capture
  const uint64_t f0 = h->fwd_tasks, b0 = h->bwd_tasks, l0 = h->launches;
  if (hipStreamBeginCapture(h->st, hipStreamCaptureModeThreadLocal) != hipSuccess)
    return fail(STAGE_E_DEVICE, "hipStreamBeginCapture failed");
  int rc = STAGE_OK;
  h->capturing = true;
  if (zero_grads_first) rc = stage_zero_grads(h);
  if (rc == STAGE_OK) rc = stage_run_schedule(h, M, K, order, xs, dys, ys, dxs, auxs, explicit_ops, n_ops);
  h->capturing = false;
  hipGraph_t g = nullptr;
  hipError_t e = hipStreamEndCapture(h->st, &g);   // always: the stream must leave capture mode
  h->graph_fwd = h->fwd_tasks - f0; h->graph_bwd = h->bwd_tasks - b0; h->graph_launches = h->launches - l0;
  h->fwd_tasks = f0; h->bwd_tasks = b0; h->launches = l0;   // captured, not run
  if (rc != STAGE_OK) { if (g) (void)hipGraphDestroy(g); return rc; }
  if (e != hipSuccess || !g) return fail(STAGE_E_DEVICE, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
  h->graph = g;
  e = hipGraphInstantiate(&h->graph_exec, g, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    h->graph_exec = nullptr;
    return fail(STAGE_E_DEVICE, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
  }
  return STAGE_OK;
}

int stage_graph_launch(stage_handle h) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (!h->graph_exec) return fail(STAGE_E_BAD_ORDER, "no captured iteration: call stage_graph_capture first");
  if (h->live != 0) return fail(STAGE_E_BAD_ORDER, "%d micro-batches are still resident", h->live);
  hipError_t e = hipGraphLaunch(h->graph_exec, h->st);
  if (e != hipSuccess) return fail(STAGE_E_DEVICE, "hipGraphLaunch failed: %s", hipGetErrorString(e));
  h->fwd_tasks += h->graph_fwd; h->bwd_tasks += h->graph_bwd; h->launches += h->graph_launches;
  return STAGE_OK;
}

int stage_stream(stage_handle h, void** hip_stream_out) {
  if (!h || !hip_stream_out) return fail(STAGE_E_NULL, "handle and hip_stream_out must not be NULL");
  *hip_stream_out = (void*)h->st;
  return STAGE_OK;
}

int stage_get_config(stage_handle h, stage_config* cfg_out) {
  if (!h || !cfg_out) return fail(STAGE_E_NULL, "handle and cfg_out must not be NULL");
  *cfg_out = h->cfg;
  return STAGE_OK;
}

int stage_grads(stage_handle h, void** grads_dev, uint64_t* n) {
  if (!h || !grads_dev || !n) return fail(STAGE_E_NULL, "handle, grads_dev and n must not be NULL");
  *grads_dev = h->grads;
  *n = h->L.n_params;
  return STAGE_OK;
}

int stage_zero_grads(stage_handle h) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  return h->run(KC_COPY, 0, [&](hipStream_t q) { return launch_zero(h->grads, h->L.grad_bytes, q); });
}

int stage_apply_adam(stage_handle h, void* weights_dev, float* master_dev, float* m_dev, float* v_dev, int step, float lr,
                     float beta1, float beta2, float eps, float grad_scale, int zero_grads) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (step < 1) return fail(STAGE_E_CONFIG, "step counts from 1 (got %d)", step);
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f))
    return fail(STAGE_E_CONFIG, "beta1 and beta2 must lie in [0, 1) and eps must be positive");
  if (h->live != 0) return fail(STAGE_E_BAD_ORDER, "%d micro-batches are still resident: the update belongs after the iteration", h->live);
  if (h->dry) { ++h->launches; return STAGE_OK; }
  if (!weights_dev || !master_dev || !m_dev || !v_dev) return fail(STAGE_E_NULL, "weights, master weights and both moments must not be NULL");
  if (weights_dev != (const void*)h->W) return fail(STAGE_E_CONFIG, "weights_dev must be the weights buffer given to stage_init");
  if (((uintptr_t)master_dev | (uintptr_t)m_dev | (uintptr_t)v_dev) % 16) return fail(STAGE_E_CONFIG, "fp32 state must be 16-byte aligned");
  const double c1 = 1.0 / (1.0 - std::pow((double)beta1, step)), c2 = 1.0 / (1.0 - std::pow((double)beta2, step));
  return h->run(KC_COPY, 0, [&](hipStream_t q) {
    return launch_adam(h->dt, h->grads, master_dev, m_dev, v_dev, weights_dev, h->L.n_params, lr, beta1, beta2, eps,
                       (float)c1, (float)c2, grad_scale, zero_grads, q);
  });
}

int stage_stats(stage_handle h, stage_stats_t* out) {
  if (!h || !out) return fail(STAGE_E_NULL, "handle and out must not be NULL");
  out->slot_bytes = h->L.slot_bytes;
  out->peak_activation_bytes = (uint64_t)h->peak_live * h->L.slot_bytes +
                               (h->L.recompute ? (uint64_t)(1 + h->L.ws_copies) * h->L.act_bytes : 0);
  out->live_slots = h->live;
  out->peak_live_slots = h->peak_live;
  out->fwd_tasks = h->fwd_tasks;
  out->bwd_tasks = h->bwd_tasks;
  out->kernel_launches = h->launches;
  return STAGE_OK;
}

int stage_reset_stats(stage_handle h) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  h->peak_live = h->live;
  h->fwd_tasks = h->bwd_tasks = h->launches = 0;
  return STAGE_OK;
}

int stage_profile_enable(stage_handle h, int on) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (!h->dry && (hipStreamSynchronize(h->st) != hipSuccess || hipStreamSynchronize(h->side) != hipSuccess))
    return fail(STAGE_E_DEVICE, "stream synchronise failed");
  h->profiling = on != 0;
  h->events_used = 0;
  return STAGE_OK;
}

int stage_profile_read(stage_handle h, int n, uint64_t* launches, double* ms, double* flops) {
  if (!h || !launches || !ms || !flops) return fail(STAGE_E_NULL, "arguments must not be NULL");
  if (!h->dry && (hipStreamSynchronize(h->st) != hipSuccess || hipStreamSynchronize(h->side) != hipSuccess))
    return fail(STAGE_E_DEVICE, "stream synchronise failed");
  if (!h->dry && h->fwd && (hipStreamSynchronize(h->fwd) != hipSuccess || (h->bwd2 && hipStreamSynchronize(h->bwd2) != hipSuccess)))
    return fail(STAGE_E_DEVICE, "stream synchronise failed");
  for (int i = 0; i < n; ++i) { launches[i] = 0; ms[i] = 0; flops[i] = 0; }
  for (size_t i = 0; i < h->events_used; ++i) {
    const ProfEvent& e = h->events[i];
    if (e.cls >= n) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, e.a, e.b) != hipSuccess) return fail(STAGE_E_DEVICE, "hipEventElapsedTime failed");
    launches[e.cls] += 1; ms[e.cls] += t; flops[e.cls] += e.flops;
  }
  h->events_used = 0;
  return STAGE_OK;
}

int stage_profile_launches(stage_handle h, stage_launch_record* out, int capacity) {
  if (!h || !out) return fail(STAGE_E_NULL, "handle and out must not be NULL");
  if (!h->dry) {
    hipError_t e = hipStreamSynchronize(h->st);
    if (e == hipSuccess) e = hipStreamSynchronize(h->side);
    if (e == hipSuccess && h->fwd) e = hipStreamSynchronize(h->fwd);
    if (e == hipSuccess && h->bwd2) e = hipStreamSynchronize(h->bwd2);
    if (e != hipSuccess) return fail(STAGE_E_DEVICE, "stream synchronise failed: %s", hipGetErrorString(e));
  }
  int n = 0;
  for (size_t i = 0; i < h->events_used && n < capacity; ++i, ++n) {
    const ProfEvent& e = h->events[i];
    float t = 0.f;
    if (hipEventElapsedTime(&t, e.a, e.b) != hipSuccess) return fail(STAGE_E_DEVICE, "hipEventElapsedTime failed");
    out[n] = stage_launch_record{e.cls, e.lane, e.M, e.N, e.K, e.batch, (double)t, e.flops};
  }
  return n;
}

const char* stage_profile_class_name(int i) { return (i >= 0 && i < KC_COUNT) ? kClassNames[i] : nullptr; }

int stage_sync(stage_handle h) {
  if (!h) return fail(STAGE_E_NULL, "handle is NULL");
  if (h->dry) return STAGE_OK;
  hipError_t e = hipStreamSynchronize(h->st);
  if (e == hipSuccess) e = hipStreamSynchronize(h->side);
  if (e != hipSuccess) return fail(STAGE_E_DEVICE, "stream synchronise failed: %s", hipGetErrorString(e));
  if (h->cfg.has_mlm_head) {
    int32_t info[2] = {0, 0};
    if (hipMemcpy(info, h->ws(h->L.wh_info), 8, hipMemcpyDeviceToHost) != hipSuccess)
      return fail(STAGE_E_DEVICE, "hipMemcpy failed");
    for (int c = 0; h->L.recompute && !info[1] && c < h->L.ws_copies; ++c)
      if (hipMemcpy(info, h->ws((size_t)c * h->L.workspace_bytes + h->L.wh_info2), 8, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(STAGE_E_DEVICE, "hipMemcpy failed");
    if (info[1]) return fail(STAGE_E_CONFIG, "a micro-batch predicted more rows than mlm_max_rows; the surplus was dropped");
  }
  return STAGE_OK;
}

}  // extern "C"
