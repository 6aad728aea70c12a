// C ABI of the d2Cache selective-refresh step (see include/d2c.h): argument
// validation, workspace ownership and the order of kernel launches.  No
// arithmetic of the method lives here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/d2c.h"
#include "../../include/d2c_tools.h"
#include "internal.h"

using namespace d2c;

bool d2c::set_tunable(Tunables& t, const char* name, int value) {
  if (!strcmp(name, "gemm_target_wgs")) t.gemm_target_wgs = value;
  else if (!strcmp(name, "gemm_max_splits")) t.gemm_max_splits = std::max(1, std::min(8, value));
  else if (!strcmp(name, "gemm_nt_big_n")) t.gemm_nt_big_n = value;
  else if (!strcmp(name, "gemm_wide_tiles")) t.gemm_wide_tiles = value;
  else if (!strcmp(name, "gemm_wide_mt")) t.gemm_wide_mt = (value >= 6 && value <= 8) ? value : 0;
  else if (!strcmp(name, "gemm_wide_min_rows")) t.gemm_wide_min_rows = value;
  else if (!strcmp(name, "gemm_tall_chunk")) t.gemm_tall_chunk = value;
  else if (!strcmp(name, "gemm_waves")) t.gemm_waves = (value == 8 || value == 4 || value == 6 || value == 7 || value == 10) ? value : 0;
  else if (!strcmp(name, "gemm_preshuffle")) t.gemm_preshuffle = value != 0;
  else if (!strcmp(name, "gemm_rot")) t.gemm_rot = value < 0 ? 0 : value;
  else if (!strcmp(name, "attn_tiled_min_m")) t.attn_tiled_min_m = value < 1 ? 1 : value;
  else if (!strcmp(name, "attn_max_splits")) t.attn_max_splits = std::max(1, std::min(8, value));
  else if (!strcmp(name, "attn_qt")) t.attn_qt = value == 1 ? 1 : value == 2 ? 2 : 0;
  else if (!strcmp(name, "attn_waves")) t.attn_waves = value == 4 ? 4 : value == 8 ? 8 : 0;
  else if (!strcmp(name, "attn_target_wgs")) t.attn_target_wgs = std::max(1, value);
  else if (!strcmp(name, "side_stream")) t.side_stream = value != 0;
  else return false;
  return true;
}

// ---- d2c_select_static: Eq. 1's per-chunk (max, argmax, sum) triples live in this file-scope device array
// instead of a context's workspace, so the call needs no context and never allocates.  Each GPU holds its
// own copy of the array at its own address; the address is looked up once per device.
constexpr int kStaticMaxRows = D2C_STATIC_MAX_ROWS;
constexpr size_t kStaticFloats = (size_t)kStaticMaxRows * 64 * 3;        // 64 = most chunks per vocabulary row
static __device__ __align__(256) float scratch[kStaticFloats];

struct d2c_ctx {
  d2c_dims dims{};
  Tunables tun;                 // this context's launch-shape tunables
  int device = 0;
  int64_t pre_bytes = 0;        // library-owned pre-tiled weight copies
  int64_t rollout_bytes = 0;    // head averages, per-head probability rows, chain scratch, rollout block
  int64_t attn_scratch_bytes = 0;
  // borrowed weights
  const void* tok_emb = nullptr;
  const float* final_norm = nullptr;
  const void* lm_head = nullptr;
  std::vector<const float*> attn_norm, bqkv, ffn_norm;
  std::vector<const void*> wqkv, wo, w_gate_up, w_down;
  // pre = the projection matrices above (and lm_head) point at library-owned pre-tiled copies made by
  // d2c_init (16-row x 256-byte blocks in the order the projection kernel's waves load them)
  bool pre = false;
  // fused_swiglu = the pre-tiled gate/up copies alternate gate and up tiles and the projection applies
  // the SwiGLU in its epilogue (no partials, no separate launch)
  bool fused_swiglu = false;
  // workspace (device)
  std::vector<void*> allocs;
  int64_t ws_bytes = 0;
  float* hidden = nullptr;      // [max_rows, d]
  void* a_norm = nullptr;       // T [max_seq, d]
  void* q = nullptr;            // T [n_layers, max_seq, d_q]: one slot per layer (a second stream may read it later)
  void* attn_o = nullptr;       // T [max_seq, d_q]
  void* act = nullptr;          // T [max_seq, F]
  float* lse = nullptr;         // [n_layers, H, max_seq]
  float* attn_part = nullptr;   // scratch of the LDS-tiled attention: split partials, unnormalised probabilities, references
  size_t attn_part_floats = 0;
  float* partial = nullptr;     // split partials of the current projection
  size_t partial_floats = 0;
  float* roll = nullptr;        // d2c_refresh_layer: the rollout block after the layer, [max_seq, max_seq]
  // d2c_step keeps every layer's head average (per batch slot: [n_layers][max_seq * max_seq]) and turns
  // them into the influence scores by a row-vector chain after the last layer
  float* abar_all = nullptr;
  // per-head attention rows (bf16) of the few-row attention launches, [max_batch][n_layers][probs_elems]
  uint16_t* probs_all = nullptr;
  float* chain_u = nullptr;     // [n_layers, max_seq]: the chain's per-layer vectors (one sequence at a time)
  float* chain_g = nullptr;     // [n_layers, max_seq * max_seq]: the dense m x m blocks of the chain
  size_t probs_elems = 0;
  int max_batch = 1;            // sequences whose rows d2c_step projects together
  size_t max_rows = 0;          // max_seq * max_batch: rows the row-count-sized buffers hold
  void* head_a = nullptr;       // T [head_rows, d]
  float* logits = nullptr;      // [head_rows, vocab]
  float* conf_part = nullptr;   // per-chunk (max, argmax, sum) triples of Eq. 1 for up to max_seq rows
  int head_rows = 0;
  float* rope_cos = nullptr;    // [max_seq, head_dim/2]
  float* rope_sin = nullptr;
  // The head-averaged attention rows and the rollout only feed the selection at the end of a step.  With
  // the side_stream tunable on, d2c_step runs them on a second stream beside the projections: fwd_done[l] is
  // recorded on the caller's stream after layer l's attention, side_done on the side stream after the last
  // rollout update.  Off (the default: two busy queues slow every launch down) they queue on the caller's.
  hipStream_t side = nullptr;
  std::vector<hipEvent_t> fwd_done;
  hipEvent_t side_done = nullptr;
  int32_t* counts_host = nullptr;   // pinned
  int counts_host_cap = 0;
  // optional per-launch timing with HIP events (d2c_profile_begin / d2c_profile_end)
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;  // start/stop pairs
  std::vector<int> prof_cls;
  std::vector<double> prof_bytes;
  size_t prof_used = 0;
  std::string err;
};

namespace {

std::string g_init_err;

int fail(d2c_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg; else g_init_err = msg;
  return code;
}

constexpr int kStaticMaxDevices = 64;
float* g_static_ptr[kStaticMaxDevices] = {};
std::mutex g_static_mu;

// Device address of this GPU's copy of `scratch` (the array's name is only a host-side handle).
int static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(nullptr, D2C_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kStaticMaxDevices) return fail(nullptr, D2C_ESHAPE, "device ordinal beyond the static table");
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return fail(nullptr, D2C_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    }
    g_static_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_static_ptr[dev];
  return D2C_OK;
}


#define D2C_HIP(ctx, expr)                                                                  \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail(ctx, D2C_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_));        \
  } while (0)

constexpr size_t kProfMaxPairs = 1 << 17;

// Records a start event for one launch of class cls; returns the pair's slot or -1.
int prof_start(d2c_ctx* c, hipStream_t st, int cls, double bytes) {
  if (!c->prof_on || c->prof_used >= kProfMaxPairs) return -1;
  const size_t slot = c->prof_used;
  if (c->prof_ev.size() < 2 * (slot + 1)) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return -1;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return -1; }
    c->prof_ev.push_back(a);
    c->prof_ev.push_back(b);
    c->prof_cls.push_back(0);
    c->prof_bytes.push_back(0.0);
  }
  c->prof_cls[slot] = cls;
  c->prof_bytes[slot] = bytes;
  if (hipEventRecord(c->prof_ev[2 * slot], st) != hipSuccess) return -1;
  c->prof_used = slot + 1;
  return (int)slot;
}
void prof_stop(d2c_ctx* c, hipStream_t st, int slot) {
  if (slot >= 0) (void)hipEventRecord(c->prof_ev[2 * (size_t)slot + 1], st);
}

#define D2C_TIMED(ctx, st, cls, nbytes, expr)              \
  do {                                                     \
    const int slot_ = prof_start(ctx, st, cls, nbytes);    \
    D2C_HIP(ctx, expr);                                    \
    prof_stop(ctx, st, slot_);                             \
  } while (0)

template <typename P>
int ws_alloc(d2c_ctx* ctx, P** out, size_t bytes) {
  void* p = nullptr;
  if (bytes == 0) bytes = 256;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, D2C_ENOMEM, "hipMalloc of " + std::to_string(bytes) + " bytes failed: " + hipGetErrorString(e));
  }
  ctx->allocs.push_back(p);
  ctx->ws_bytes += (int64_t)bytes;
  *out = reinterpret_cast<P*>(p);
  return D2C_OK;
}

size_t tsize(const d2c_ctx* c) { return dtype_size(c->dims.dtype); }
int d_q(const d2c_ctx* c) { return c->dims.n_heads * c->dims.head_dim; }
int d_kv(const d2c_ctx* c) { return c->dims.n_kv_heads * c->dims.head_dim; }

int pre_chunks(const d2c_ctx* c, int K) { return (int)(((size_t)K * tsize(c) + 255) / 256); }

// One projection on m rows: P = A W^T as split partials in the context's buffer.  W is one of the
// context's own projection matrices (pre-tiled when c->pre).
int project(d2c_ctx* c, const void* A, int lda, const void* W, int m, int N, int K, GemmPlan* plan_out,
            size_t* stride_out, hipStream_t st, bool single_split = false, float* dst = nullptr) {
  GemmPlan pl = plan_gemm(c->tun, c->dims.dtype, m, N, K, single_split);
  const size_t stride = (size_t)m * N;
  float* P = dst ? dst : c->partial;
  if (!dst && stride * pl.splits > c->partial_floats) return fail(c, D2C_ESHAPE, "projection partials exceed workspace");
  D2C_TIMED(c, st, D2C_PROF_GEMM, (double)N * K * tsize(c),
            launch_gemm(c->dims.dtype, pl, A, lda, W, c->pre ? pre_chunks(c, K) : K, P, N, stride, m, N, K, st,
                        c->pre));
  *plan_out = pl;
  *stride_out = stride;
  return D2C_OK;
}

// One sequence's share of a block: its m selected rows sit at rows off .. off+m of the compact buffers.
struct Seg {
  const int32_t* idx;
  int m, off;
  void *k_cache, *v_cache;      // this layer's cache of the sequence
  int L;
  float* abar;                  // [m, L] out: head average of this layer (null = not wanted)
  void* probs;                  // bf16 [H, m, L] out: per-head attention rows written by the attention launch
                                // itself (null = not wanted; only where attention_fwd_emits_probs)
  const float* roll_in;         // rollout block before this layer (ignored at layer 0)
  float* roll_out;              // rollout block after it; null = no rollout update
};

// One block on the M = sum of m compact rows of n_seg sequences.  The projections run once over all M rows
// (the weights are streamed once for the whole batch); RoPE + cache update, attention, the head average and
// the rollout run per sequence on its slice.  a_ready: ctx->a_norm already holds RMSNorm(hidden) *
// attn_norm[layer].  next_gain: when non-null the last kernel also leaves RMSNorm(hidden) * next_gain in
// ctx->a_norm.
// side: the stream the head average and the rollout update run on; when it differs from st they are
// ordered after this layer's attention by ctx->fwd_done[layer] and the caller joins them later.
int layer_impl(d2c_ctx* c, int layer, float* hidden, const Seg* segs, int n_seg, int M, bool a_ready,
               const float* next_gain, hipStream_t st, hipStream_t side, bool record_fwd = false) {
  const d2c_dims& D = c->dims;
  const int dt = D.dtype, d = D.d_model, dq = d_q(c), dkv = d_kv(c), F = D.d_ffn;
  const size_t ts = tsize(c);
  char* q = (char*)c->q + (size_t)layer * c->max_rows * dq * ts;
  float* lse = c->lse + (size_t)layer * D.n_heads * c->max_rows;
  GemmPlan pl;
  size_t stride;
  int rc;
  if (!a_ready)
    D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
              launch_add_norm(dt, hidden, nullptr, 0, 0, d, M, d, c->attn_norm[layer], D.rms_eps, c->a_norm, st));
  if ((rc = project(c, c->a_norm, d, c->wqkv[layer], M, dq + 2 * dkv, d, &pl, &stride, st)) != D2C_OK) return rc;
  // RoPE and cache update per sequence; the few-row attention per sequence as well, the LDS-tiled attention of
  // the sequences with many rows in batched launches (they write the head average themselves, on this stream)
  std::vector<TiledCall> tiled;
  double tiled_bytes = 0.0;
  auto flush_tiled = [&]() -> int {
    if (tiled.empty()) return D2C_OK;
    D2C_TIMED(c, st, D2C_PROF_ATTENTION, tiled_bytes,
              launch_attention_tiled(c->tun, tiled.data(), (int)tiled.size(), D.n_heads, D.n_kv_heads, D.head_dim,
                                     c->attn_part, c->attn_part_floats, st));
    tiled.clear();
    tiled_bytes = 0.0;
    return D2C_OK;
  };
  // RoPE + cache update of consecutive non-empty slices in one launch (their rows are consecutive in the
  // compact buffers; an empty slice in between does not break the run)
  {
    std::vector<RopeCall> ropes;
    auto flush_rope = [&]() -> int {
      if (ropes.empty()) return D2C_OK;
      const int off0 = ropes[0].off;
      for (auto& rcall : ropes) rcall.off -= off0;
      D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
                launch_qkv_rope_scatter(dt, c->partial + (size_t)off0 * (dq + 2 * dkv), pl.splits, stride, dq + 2 * dkv,
                                        c->bqkv.empty() ? nullptr : c->bqkv[layer], ropes.data(), (int)ropes.size(),
                                        D.n_heads, D.n_kv_heads, D.head_dim, c->rope_cos, c->rope_sin,
                                        q + (size_t)off0 * dq * ts, st));
      ropes.clear();
      return D2C_OK;
    };
    for (int b = 0; b < n_seg; ++b) {
      const Seg& g = segs[b];
      if (g.m <= 0) continue;
      ropes.push_back(RopeCall{g.idx, g.k_cache, g.v_cache, g.off, g.m});
      if ((int)ropes.size() == rope_max_batch() && (rc = flush_rope())) return rc;
    }
    if ((rc = flush_rope())) return rc;
  }
  for (int b = 0; b < n_seg; ++b) {
    const Seg& g = segs[b];
    if (g.m <= 0) continue;
    void* qb = q + (size_t)g.off * dq * ts;
    void* ob = (char*)c->attn_o + (size_t)g.off * dq * ts;
    float* lb = lse + (size_t)D.n_heads * g.off;
    if (attention_is_tiled(c->tun, dt, g.m, g.L)) {
      tiled.push_back(TiledCall{qb, g.k_cache, g.v_cache, g.m, g.L, ob, lb, g.abar});
      tiled_bytes += 2.0 * g.L * dkv * ts;
      if ((int)tiled.size() == attention_tiled_max_batch() && (rc = flush_tiled())) return rc;
    } else {
      D2C_TIMED(c, st, D2C_PROF_ATTENTION, 2.0 * g.L * dkv * ts,
                launch_attention_fwd(c->tun, dt, qb, g.k_cache, g.v_cache, g.m, g.L, D.n_heads, D.n_kv_heads, D.head_dim,
                                     ob, lb, c->attn_part, c->attn_part_floats, st, g.probs, nullptr));
    }
  }
  if ((rc = flush_tiled())) return rc;
  // what is left for the second stream: the second pass of the few-row kernels and the rollout update
  bool any_side = false;
  for (int b = 0; b < n_seg; ++b)
    any_side = any_side || (segs[b].m > 0 && segs[b].abar &&
                            (!attention_is_tiled(c->tun, dt, segs[b].m, segs[b].L) || segs[b].roll_out));
  if (record_fwd && !any_side && side != st) D2C_HIP(c, hipEventRecord(c->fwd_done[layer], st));
  if (any_side) {
    if (side != st) {
      D2C_HIP(c, hipEventRecord(c->fwd_done[layer], st));
      D2C_HIP(c, hipStreamWaitEvent(side, c->fwd_done[layer], 0));
    }
    for (int b = 0; b < n_seg; ++b) {
      const Seg& g = segs[b];
      if (g.m <= 0 || !g.abar) continue;
      if (!attention_is_tiled(c->tun, dt, g.m, g.L))
        D2C_TIMED(c, side, D2C_PROF_ATTN_AVG, 0.0,
                  launch_attention_avg(c->tun, dt, q + (size_t)g.off * dq * ts, g.k_cache, lse + (size_t)D.n_heads * g.off,
                                       g.m, g.L, D.n_heads, D.n_kv_heads, D.head_dim, g.abar, side));
      if (g.roll_out)
        D2C_TIMED(c, side, D2C_PROF_ROLLOUT, 0.0,
                  launch_rollout(g.abar, g.roll_in, g.roll_out, g.idx, g.m, g.L, layer == 0, side));
    }
  }
  if ((rc = project(c, c->attn_o, dq, c->wo[layer], M, d, dq, &pl, &stride, st)) != D2C_OK) return rc;
  D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
            launch_add_norm(dt, hidden, c->partial, pl.splits, stride, d, M, d, c->ffn_norm[layer], D.rms_eps,
                            c->a_norm, st));
  if (c->fused_swiglu) {
    pl = plan_gemm(c->tun, dt, M, 2 * F, d, true);
    D2C_TIMED(c, st, D2C_PROF_GEMM, 2.0 * F * d * tsize(c),
              launch_gemm_swiglu(dt, pl, c->a_norm, d, c->w_gate_up[layer], pre_chunks(c, d), c->act, F, M, d, st));
  } else {
    if ((rc = project(c, c->a_norm, d, c->w_gate_up[layer], M, 2 * F, d, &pl, &stride, st)) != D2C_OK) return rc;
    D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
              launch_swiglu(dt, c->partial, pl.splits, stride, 2 * F, M, F, c->act, st));
  }
  if ((rc = project(c, c->act, F, c->w_down[layer], M, d, F, &pl, &stride, st)) != D2C_OK) return rc;
  D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
            launch_add_norm(dt, hidden, c->partial, pl.splits, stride, d, M, d, next_gain, D.rms_eps,
                            next_gain ? c->a_norm : nullptr, st));
  return D2C_OK;
}

int check_idx_host(d2c_ctx* c, const int32_t* idx_host, int m, int L) {
  if (m < 0 || L <= 0 || m > L) return fail(c, D2C_EINVAL, "need 0 <= m <= L");
  if (L > c->dims.max_seq) return fail(c, D2C_ESHAPE, "L exceeds max_seq of the context");
  if (m > 0 && !idx_host) return fail(c, D2C_EINVAL, "idx_host is null");
  for (int r = 0; r < m; ++r) {
    if (idx_host[r] < 0 || idx_host[r] >= L) return fail(c, D2C_EINVAL, "idx out of range");
    if (r && idx_host[r] <= idx_host[r - 1]) return fail(c, D2C_EINVAL, "idx must be ascending and distinct");
  }
  return D2C_OK;
}

int check_params(d2c_ctx* c, const d2c_params* p) {
  if (!p) return fail(c, D2C_EINVAL, "params is null");
  if (!(p->sigma > 0.f) || p->k < 0 || p->block_len <= 0 || p->n_unmask < 0 || !(p->p >= 0.f) ||
      (p->cand_mode != 0 && p->cand_mode != 1) || !(p->threshold >= 0.f) ||
      (p->conf_decode != 0 && p->conf_decode != 1) || p->rollout_layers < 0)
    return fail(c, D2C_EINVAL, "bad selection parameters");
  return D2C_OK;
}

// Floats of split partials, attention partials and head-average partials that the launch plans can ask for
// under tunables t, over every row count and sequence length the context admits.
struct WsNeeds { size_t partial, attn_part; };
WsNeeds ws_needs(const d2c_dims& D, size_t max_rows, const Tunables& t) {
  const int dq = D.n_heads * D.head_dim, dkv = D.n_kv_heads * D.head_dim;
  const int shapes[4][2] = {{dq + 2 * dkv, D.d_model}, {D.d_model, dq}, {2 * D.d_ffn, D.d_model}, {D.d_model, D.d_ffn}};
  WsNeeds n{0, 0};
  for (int m = 1; m <= (int)max_rows; ++m)
    for (auto& s : shapes) {
      // up to 128 rows leave room for the largest split count; beyond that the planner's choice is taken
      const GemmPlan pl = plan_gemm(t, D.dtype, m, s[0], s[1]);
      n.partial = std::max(n.partial, (size_t)(m <= 128 ? 8 : pl.splits) * m * s[0]);
    }
  // one piece per sequence of a batched attention launch
  const int batch = std::max(1, std::min((int)(max_rows / (size_t)D.max_seq), attention_tiled_max_batch()));
  n.attn_part = (size_t)batch * attention_scratch_floats(t, D.dtype, D.max_seq, D.max_seq, D.n_heads, D.head_dim);
  return n;
}

}  // namespace

extern "C" {

int d2c_init(const d2c_dims* dims, const d2c_weights* w, d2c_ctx** out) { return d2c_init_tuned(dims, w, nullptr, 0, out); }

int d2c_init_tuned(const d2c_dims* dims, const d2c_weights* w, const d2c_tunable* tun, int32_t n_tun, d2c_ctx** out) {
  if (!dims || !w || !out) return fail(nullptr, D2C_EINVAL, "null argument");
  if (n_tun < 0 || (n_tun > 0 && !tun)) return fail(nullptr, D2C_EINVAL, "bad tunable list");
  Tunables tn;
  for (int i = 0; i < n_tun; ++i)
    if (!tun[i].name || !set_tunable(tn, tun[i].name, tun[i].value))
      return fail(nullptr, D2C_EINVAL, std::string("unknown tunable ") + (tun[i].name ? tun[i].name : "(null)"));
  const d2c_dims& D = *dims;
  if (D.n_layers <= 0 || D.d_model <= 0 || D.n_heads <= 0 || D.n_kv_heads <= 0 || D.head_dim <= 0 || D.d_ffn <= 0 ||
      D.vocab <= 0 || D.max_seq <= 0)
    return fail(nullptr, D2C_EINVAL, "dimensions must be positive");
  if (D.dtype != D2C_F32 && D.dtype != D2C_BF16) return fail(nullptr, D2C_EINVAL, "dtype must be D2C_F32 or D2C_BF16");
  if (D.n_heads % D.n_kv_heads) return fail(nullptr, D2C_EINVAL, "n_heads must be a multiple of n_kv_heads");
  if (D.head_dim % 2) return fail(nullptr, D2C_EINVAL, "head_dim must be even");
  if (D.dtype == D2C_BF16 && D.head_dim != 64 && D.head_dim != 128)
    return fail(nullptr, D2C_ESHAPE, "bf16 attention supports head_dim 64 or 128");
  const int e = D.dtype == D2C_BF16 ? 8 : 4;
  if (D.d_model % e || D.d_ffn % e || (D.n_heads * D.head_dim) % e)
    return fail(nullptr, D2C_ESHAPE, "d_model, d_ffn and n_heads*head_dim must be multiples of 16 bytes of T");
  if (D.max_seq > select_max_len()) return fail(nullptr, D2C_ESHAPE, "max_seq exceeds the selection kernel's limit");
  if (D.max_batch < 0 || D.max_batch > 64) return fail(nullptr, D2C_EINVAL, "max_batch must be in [0, 64]");
  if (D.mask_id < 0 || D.mask_id >= D.vocab) return fail(nullptr, D2C_EINVAL, "mask_id outside the vocabulary");
  if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
      !w->w_gate_up || !w->w_down)
    return fail(nullptr, D2C_EINVAL, "null weight pointer");
  for (int l = 0; l < D.n_layers; ++l)
    if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate_up[l] || !w->w_down[l] ||
        (w->bqkv && !w->bqkv[l]))
      return fail(nullptr, D2C_EINVAL, "null per-layer weight pointer");

  d2c_ctx* c = new (std::nothrow) d2c_ctx();
  if (!c) return fail(nullptr, D2C_ENOMEM, "out of host memory");
  c->dims = D;
  c->tun = tn;
  c->tok_emb = w->tok_emb; c->final_norm = w->final_norm; c->lm_head = w->lm_head;
  for (int l = 0; l < D.n_layers; ++l) {
    c->attn_norm.push_back(w->attn_norm[l]); c->wqkv.push_back(w->wqkv[l]); c->wo.push_back(w->wo[l]);
    c->ffn_norm.push_back(w->ffn_norm[l]); c->w_gate_up.push_back(w->w_gate_up[l]); c->w_down.push_back(w->w_down[l]);
    if (w->bqkv) c->bqkv.push_back(w->bqkv[l]);
  }
  int rc = D2C_OK;
  auto bail = [&](int code) { std::string m = c->err; d2c_destroy(c); g_init_err = m; return code; };
  if (hipGetDevice(&c->device) != hipSuccess) return bail(fail(c, D2C_EHIP, "hipGetDevice failed"));

  c->max_batch = std::max(1, (int)D.max_batch);
  c->max_rows = (size_t)D.max_seq * c->max_batch;
  const size_t ts = tsize(c), Lm = (size_t)D.max_seq, Lr = c->max_rows, d = (size_t)D.d_model, dq = (size_t)d_q(c),
               F = (size_t)D.d_ffn;
  const WsNeeds need = ws_needs(D, Lr, c->tun);
  const size_t pf = need.partial;
  c->partial_floats = pf;
  c->head_rows = (int)std::min<size_t>(Lm, 256);
  c->attn_part_floats = need.attn_part;
  const int64_t ws0 = c->ws_bytes;
  if ((rc = ws_alloc(c, &c->roll, Lm * Lm * 4)) ||
      (rc = ws_alloc(c, &c->abar_all, (size_t)c->max_batch * D.n_layers * Lm * Lm * 4)))
    return bail(rc);
  c->probs_elems = attention_probs_elems(D.dtype, D.n_heads, D.max_seq);
  if ((rc = ws_alloc(c, &c->probs_all, (size_t)c->max_batch * D.n_layers * c->probs_elems * 2)) ||
      (rc = ws_alloc(c, &c->chain_u, (size_t)D.n_layers * Lm * 4)) ||
      (rc = ws_alloc(c, &c->chain_g, (size_t)D.n_layers * Lm * Lm * 4)))
    return bail(rc);
  c->rollout_bytes = c->ws_bytes - ws0;
  c->attn_scratch_bytes = (int64_t)std::max<size_t>(1, c->attn_part_floats) * 4;
  if ((rc = ws_alloc(c, &c->hidden, Lr * d * 4)) || (rc = ws_alloc(c, &c->a_norm, Lr * d * ts)) ||
      (rc = ws_alloc(c, &c->q, (size_t)D.n_layers * Lr * dq * ts)) || (rc = ws_alloc(c, &c->attn_o, Lr * dq * ts)) ||
      (rc = ws_alloc(c, &c->act, Lr * F * ts)) ||
      (rc = ws_alloc(c, &c->lse, (size_t)D.n_layers * D.n_heads * Lr * 4)) ||
      (rc = ws_alloc(c, &c->attn_part, std::max<size_t>(1, c->attn_part_floats) * 4)) ||
      (rc = ws_alloc(c, &c->partial, pf * 4)) ||
      (rc = ws_alloc(c, &c->head_a, (size_t)c->head_rows * d * ts)) ||
      (rc = ws_alloc(c, &c->logits, (size_t)c->head_rows * D.vocab * 4)) ||
      (rc = ws_alloc(c, &c->conf_part, confidence_scratch_floats(D.max_seq) * 4)) ||
      (rc = ws_alloc(c, &c->rope_cos, Lm * (D.head_dim / 2) * 4)) ||
      (rc = ws_alloc(c, &c->rope_sin, Lm * (D.head_dim / 2) * 4)))
    return bail(rc);
  c->counts_host_cap = 64;
  if (hipHostMalloc((void**)&c->counts_host, sizeof(int32_t) * D2C_N_COUNTS * c->counts_host_cap) != hipSuccess)
    return bail(fail(c, D2C_ENOMEM, "hipHostMalloc failed"));
  if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess)
    return bail(fail(c, D2C_EHIP, "hipStreamCreateWithFlags failed"));
  c->fwd_done.assign(D.n_layers, nullptr);
  for (int l = 0; l < D.n_layers; ++l)
    if (hipEventCreateWithFlags(&c->fwd_done[l], hipEventDisableTiming) != hipSuccess)
      return bail(fail(c, D2C_EHIP, "hipEventCreateWithFlags failed"));
  if (hipEventCreateWithFlags(&c->side_done, hipEventDisableTiming) != hipSuccess)
    return bail(fail(c, D2C_EHIP, "hipEventCreateWithFlags failed"));
  if (c->tun.gemm_preshuffle) {
    // library-owned pre-tiled copies of every projection matrix; the caller's matrices are read here only
    // (whatever stream wrote them must be done: wait for the device once)
    if (hipDeviceSynchronize() != hipSuccess) return bail(fail(c, D2C_EHIP, "hipDeviceSynchronize failed"));
    const bool fuse = D.d_ffn % 16 == 0;
    auto retile = [&](const void*& W, int N, int K, int half = 0) -> int {
      void* dstp = nullptr;
      int rc2 = ws_alloc(c, &dstp, preshuffled_bytes(N, K, D.dtype));
      if (rc2) return rc2;
      hipError_t e = launch_preshuffle(D.dtype, W, K, N, K, dstp, nullptr, half);
      if (e != hipSuccess) return fail(c, D2C_EHIP, std::string("preshuffle: ") + hipGetErrorString(e));
      c->pre_bytes += (int64_t)preshuffled_bytes(N, K, D.dtype);
      W = dstp;
      return D2C_OK;
    };
    for (int l = 0; l < D.n_layers && !rc; ++l) {
      if ((rc = retile(c->wqkv[l], d_q(c) + 2 * d_kv(c), D.d_model)) || (rc = retile(c->wo[l], D.d_model, d_q(c))) ||
          (rc = retile(c->w_gate_up[l], 2 * D.d_ffn, D.d_model, fuse ? D.d_ffn : 0)) || (rc = retile(c->w_down[l], D.d_model, D.d_ffn)))
        break;
    }
    if (!rc) rc = retile(c->lm_head, D.vocab, D.d_model);
    if (rc) return bail(rc);
    if (hipStreamSynchronize(nullptr) != hipSuccess) return bail(fail(c, D2C_EHIP, "preshuffle failed"));
    c->pre = true;
    c->fused_swiglu = fuse;
  }
  hipError_t e2 = launch_rope_table(c->rope_cos, c->rope_sin, D.max_seq, D.head_dim, D.rope_theta, nullptr);
  if (e2 == hipSuccess) e2 = hipStreamSynchronize(nullptr);
  if (e2 != hipSuccess) return bail(fail(c, D2C_EHIP, std::string("rope table: ") + hipGetErrorString(e2)));
  *out = c;
  return D2C_OK;
}

int d2c_destroy(d2c_ctx* c) {
  if (!c) return D2C_OK;
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->counts_host) (void)hipHostFree(c->counts_host);
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->fwd_done)
    if (e) (void)hipEventDestroy(e);
  if (c->side_done) (void)hipEventDestroy(c->side_done);
  if (c->side) (void)hipStreamDestroy(c->side);
  delete c;
  return D2C_OK;
}

const char* d2c_last_error(const d2c_ctx* c) { return c ? c->err.c_str() : g_init_err.c_str(); }

int64_t d2c_workspace_bytes(const d2c_ctx* c) { return c ? c->ws_bytes : 0; }

int d2c_plan_projection(int32_t dtype, int32_t m, int32_t N, int32_t K, int32_t single_split, int32_t shape[7]) {
  if (!shape || (dtype != D2C_F32 && dtype != D2C_BF16) || m <= 0 || N <= 0 || K <= 0) return D2C_EINVAL;
  const GemmPlan pl = plan_gemm(Tunables{}, dtype, m, N, K, single_split != 0);
  const int cols = 16 * pl.nt * pl.waves;
  shape[0] = pl.mt;
  shape[1] = pl.nt;
  shape[2] = pl.waves;
  shape[3] = pl.splits;
  shape[4] = pl.k_per_split;
  shape[5] = pl.row_chunks;
  shape[6] = ((N + cols - 1) / cols) * pl.splits * pl.row_chunks;
  return D2C_OK;
}

int d2c_ctx_set_tunable(d2c_ctx* c, const char* name, int32_t value) {
  if (!c || !name) return D2C_EINVAL;
  if (!strcmp(name, "gemm_preshuffle")) return fail(c, D2C_EINVAL, "gemm_preshuffle is fixed at d2c_init_tuned");
  Tunables t = c->tun;
  if (!set_tunable(t, name, value)) return fail(c, D2C_EINVAL, std::string("unknown tunable ") + name);
  // the workspace was sized for the launch shapes of the tunables given at init: a change that asks for more is refused
  const WsNeeds need = ws_needs(c->dims, c->max_rows, t);
  if (need.partial > c->partial_floats || need.attn_part > c->attn_part_floats)
    return fail(c, D2C_ESHAPE, std::string("tunable ") + name + " needs more workspace than the context holds: pass it to d2c_init_tuned");
  c->tun = t;
  return D2C_OK;
}

int d2c_memory_info(const d2c_ctx* c, int64_t bytes[4]) {
  if (!c || !bytes) return D2C_EINVAL;
  bytes[0] = c->ws_bytes;
  bytes[1] = c->pre_bytes;
  bytes[2] = c->rollout_bytes;
  bytes[3] = c->attn_scratch_bytes;
  return D2C_OK;
}

int d2c_profile_begin(d2c_ctx* c) {
  if (!c) return D2C_EINVAL;
  c->prof_on = true;
  c->prof_used = 0;
  return D2C_OK;
}

int d2c_profile_end(d2c_ctx* c, double* ms, int64_t* launches, double* bytes) {
  if (!c) return D2C_EINVAL;
  if (!ms || !launches || !bytes) return fail(c, D2C_EINVAL, "null output");
  c->prof_on = false;
  for (int k = 0; k < D2C_PROF_CLASSES; ++k) { ms[k] = 0.0; launches[k] = 0; bytes[k] = 0.0; }
  for (size_t i = 0; i < c->prof_used; ++i) {
    D2C_HIP(c, hipEventSynchronize(c->prof_ev[2 * i + 1]));
    float t = 0.f;
    D2C_HIP(c, hipEventElapsedTime(&t, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
    const int k = c->prof_cls[i];
    ms[k] += (double)t;
    launches[k] += 1;
    bytes[k] += c->prof_bytes[i];
  }
  c->prof_used = 0;
  return D2C_OK;
}

int d2c_seq_reset(d2c_ctx* c, d2c_seq_state* s, void* stream) {
  if (!c || !s) return D2C_EINVAL;
  if (!s->tokens || !s->is_masked || !s->k_cache || !s->v_cache || !s->conf || !s->pred || !s->s_idx || !s->s_rows ||
      !s->influence || !s->mstar || !s->u_set || !s->decode_idx || !s->counts)
    return fail(c, D2C_EINVAL, "null buffer in sequence state");
  if (s->L <= 0 || s->L > c->dims.max_seq) return fail(c, D2C_ESHAPE, "L outside (0, max_seq]");
  if (s->prompt_len < 0 || s->prompt_len > s->L) return fail(c, D2C_EINVAL, "prompt_len outside [0, L]");
  hipStream_t st = (hipStream_t)stream;
  D2C_HIP(c, launch_seq_reset(s->is_masked, s->L, s->s_idx, s->s_rows, s->conf, s->pred, s->counts, st));
  D2C_HIP(c, hipMemcpyAsync(c->counts_host, s->counts, sizeof(int32_t) * D2C_N_COUNTS, hipMemcpyDeviceToHost, st));
  D2C_HIP(c, hipStreamSynchronize(st));
  s->n_s = c->counts_host[D2C_CNT_S];
  s->n_rows = c->counts_host[D2C_CNT_NEXT_ROWS];
  s->n_masked = c->counts_host[D2C_CNT_MASKED];
  s->step = 0;
  return D2C_OK;
}

int d2c_select(d2c_ctx* c, const d2c_params* p, const float* logits, const int32_t* logit_pos, int32_t n_rows,
               int32_t* tokens, uint8_t* is_masked, int32_t L, int32_t prompt_len, float* conf, int32_t* pred,
               const float* influence, int32_t* mstar, int32_t* u_set, int32_t* decode_idx, int32_t* s_next,
               int32_t* s_rows_next, int32_t* counts, float* score_out, void* stream) {
  if (!c) return D2C_EINVAL;
  int rc = check_params(c, p);
  if (rc) return rc;
  if (!tokens || !is_masked || !conf || !pred || !influence || !mstar || !u_set || !decode_idx || !s_next ||
      !s_rows_next || !counts)
    return fail(c, D2C_EINVAL, "null buffer");
  if (n_rows < 0 || (n_rows > 0 && (!logits || !logit_pos))) return fail(c, D2C_EINVAL, "logits / logit_pos missing");
  if (L <= 0 || L > c->dims.max_seq) return fail(c, D2C_ESHAPE, "L outside (0, max_seq]");
  if (prompt_len < 0 || prompt_len > L) return fail(c, D2C_EINVAL, "prompt_len outside [0, L]");
  hipStream_t st = (hipStream_t)stream;
  if (n_rows > c->dims.max_seq) return fail(c, D2C_ESHAPE, "n_rows exceeds max_seq of the context");
  D2C_HIP(c, launch_confidence(logits, logit_pos, nullptr, n_rows, c->dims.vocab, conf, pred, c->conf_part, st));
  SelectArgs a{p->sigma, p->k, p->p, p->block_len, p->n_unmask, p->cand_mode, p->threshold, p->conf_decode,
               tokens, is_masked, L, prompt_len,
               conf, pred, influence, mstar, u_set, decode_idx, s_next, s_rows_next, counts, score_out};
  D2C_HIP(c, launch_select(&a, 1, st));
  return D2C_OK;
}

int d2c_select_static(const d2c_params* p, int32_t vocab, const float* logits, const int32_t* logit_pos,
                      int32_t n_rows, int32_t* tokens, uint8_t* is_masked, int32_t L, int32_t prompt_len, float* conf,
                      int32_t* pred, const float* influence, int32_t* mstar, int32_t* u_set, int32_t* decode_idx,
                      int32_t* s_next, int32_t* s_rows_next, int32_t* counts, float* score_out, void* stream) {
  int rc = check_params(nullptr, p);
  if (rc) return rc;
  if (!tokens || !is_masked || !conf || !pred || !influence || !mstar || !u_set || !decode_idx || !s_next ||
      !s_rows_next || !counts)
    return fail(nullptr, D2C_EINVAL, "null buffer");
  if (vocab <= 0) return fail(nullptr, D2C_EINVAL, "vocab must be positive");
  if (n_rows < 0 || (n_rows > 0 && (!logits || !logit_pos))) return fail(nullptr, D2C_EINVAL, "logits / logit_pos missing");
  if (n_rows > kStaticMaxRows)
    return fail(nullptr, D2C_ESHAPE, "n_rows exceeds D2C_STATIC_MAX_ROWS (" + std::to_string(kStaticMaxRows) +
                                         "): the static scratch array holds no more");
  if (L <= 0 || L > select_max_len())
    return fail(nullptr, D2C_ESHAPE, "L outside (0, " + std::to_string(select_max_len()) + "]");
  if (prompt_len < 0 || prompt_len > L) return fail(nullptr, D2C_EINVAL, "prompt_len outside [0, L]");
  if (confidence_scratch_floats(n_rows) > kStaticFloats) return fail(nullptr, D2C_ESHAPE, "scratch array too small");
  float* sp = nullptr;
  if ((rc = static_scratch(&sp))) return rc;
  hipStream_t st = (hipStream_t)stream;
  // every (row, chunk) triple that the merge reads is written by the chunk kernel of this call: nothing in
  // the array has to start at zero, whatever the last call left there
  D2C_HIP(nullptr, launch_confidence(logits, logit_pos, nullptr, n_rows, vocab, conf, pred, sp, st));
  SelectArgs a{p->sigma, p->k, p->p, p->block_len, p->n_unmask, p->cand_mode, p->threshold, p->conf_decode,
               tokens, is_masked, L, prompt_len,
               conf, pred, influence, mstar, u_set, decode_idx, s_next, s_rows_next, counts, score_out};
  D2C_HIP(nullptr, launch_select(&a, 1, st));
  return D2C_OK;
}

int d2c_refresh_layer(d2c_ctx* c, int32_t layer, float* hidden, const int32_t* idx, const int32_t* idx_host,
                      int32_t m, void* k_cache, void* v_cache, int32_t L, float* attn_avg, float* rollout,
                      void* stream) {
  if (!c) return D2C_EINVAL;
  if (layer < 0 || layer >= c->dims.n_layers) return fail(c, D2C_EINVAL, "layer out of range");
  int rc = check_idx_host(c, idx_host, m, L);
  if (rc) return rc;
  if (m == 0) return D2C_OK;
  if (!hidden || !idx || !k_cache || !v_cache) return fail(c, D2C_EINVAL, "null buffer");
  if ((attn_avg == nullptr) != (rollout == nullptr))
    return fail(c, D2C_EINVAL, "attn_avg and rollout must both be given or both be null");
  hipStream_t st = (hipStream_t)stream;
  const Seg seg{idx, m, 0, k_cache, v_cache, L, attn_avg, nullptr, rollout, rollout ? c->roll : nullptr};
  rc = layer_impl(c, layer, hidden, &seg, 1, m, false, nullptr, st, st);
  if (rc) return rc;
  if (rollout) D2C_HIP(c, launch_copy_f32(rollout, c->roll, (size_t)m * L, st));
  return D2C_OK;
}

int d2c_attention(d2c_ctx* c, const void* q, const int32_t* idx, int32_t m, const void* new_k, const void* new_v,
                  void* k_cache, void* v_cache, int32_t L, void* out, float* attn_avg, void* stream) {
  if (!c) return D2C_EINVAL;
  if (m < 0 || L <= 0 || m > c->dims.max_seq) return fail(c, D2C_EINVAL, "bad m or L");
  if (L > c->dims.max_seq) return fail(c, D2C_ESHAPE, "L exceeds max_seq of the context");
  if (m == 0) return D2C_OK;
  if (!q || !k_cache || !v_cache || !out) return fail(c, D2C_EINVAL, "null buffer");
  if ((new_k == nullptr) != (new_v == nullptr)) return fail(c, D2C_EINVAL, "new_k and new_v go together");
  if (new_k && !idx) return fail(c, D2C_EINVAL, "idx is null");
  hipStream_t st = (hipStream_t)stream;
  const d2c_dims& D = c->dims;
  if (new_k) {
    D2C_HIP(c, launch_scatter_rows(D.dtype, new_k, k_cache, new_v, v_cache, idx, m, d_kv(c), st));
  }
  const bool tiled = attention_is_tiled(c->tun, D.dtype, m, L);
  D2C_TIMED(c, st, D2C_PROF_ATTENTION, 2.0 * L * d_kv(c) * tsize(c),
            launch_attention_fwd(c->tun, D.dtype, q, k_cache, v_cache, m, L, D.n_heads, D.n_kv_heads, D.head_dim, out, c->lse,
                                 c->attn_part, c->attn_part_floats, st, nullptr, tiled ? attn_avg : nullptr));
  if (attn_avg && !tiled)
    D2C_TIMED(c, st, D2C_PROF_ATTN_AVG, 0.0,
              launch_attention_avg(c->tun, D.dtype, q, k_cache, c->lse, m, L, D.n_heads, D.n_kv_heads, D.head_dim, attn_avg,
                                   st));
  return D2C_OK;
}

int d2c_linear(d2c_ctx* c, const void* a, const void* w, int32_t m, int32_t N, int32_t K, float* out, void* stream) {
  if (!c) return D2C_EINVAL;
  if (m < 0 || N <= 0 || K <= 0) return fail(c, D2C_EINVAL, "bad m, N or K");
  if (m > c->dims.max_seq) return fail(c, D2C_ESHAPE, "m exceeds max_seq of the context");
  if (K % (c->dims.dtype == D2C_BF16 ? 8 : 4)) return fail(c, D2C_ESHAPE, "K must be a multiple of 16 bytes of T");
  if (m == 0) return D2C_OK;
  if (!a || !w || !out) return fail(c, D2C_EINVAL, "null buffer");
  hipStream_t st = (hipStream_t)stream;
  GemmPlan pl = plan_gemm(c->tun, c->dims.dtype, m, N, K);
  const size_t stride = (size_t)m * N;
  if (stride * pl.splits > c->partial_floats) pl = plan_gemm(c->tun, c->dims.dtype, m, N, K, true);   // no room for partials
  if (pl.splits == 1) {
    D2C_TIMED(c, st, D2C_PROF_GEMM, (double)N * K * tsize(c),
              launch_gemm(c->dims.dtype, pl, a, K, w, K, out, N, stride, m, N, K, st));
    return D2C_OK;
  }
  if (stride * pl.splits > c->partial_floats) return fail(c, D2C_ESHAPE, "projection partials exceed workspace");
  D2C_TIMED(c, st, D2C_PROF_GEMM, (double)N * K * tsize(c),
            launch_gemm(c->dims.dtype, pl, a, K, w, K, c->partial, N, stride, m, N, K, st));
  D2C_HIP(c, launch_sum_splits(out, c->partial, pl.splits, stride, stride, st));
  return D2C_OK;
}

int d2c_influence(d2c_ctx* c, const float* rollout, const int32_t* idx, int32_t m, int32_t L, float* influence,
                  void* stream) {
  if (!c) return D2C_EINVAL;
  if (m < 0 || L <= 0 || m > L || !influence || (m > 0 && (!rollout || !idx))) return fail(c, D2C_EINVAL, "bad argument");
  D2C_HIP(c, launch_influence(rollout, idx, m, L, influence, (hipStream_t)stream));
  return D2C_OK;
}

int d2c_step(d2c_ctx* c, const d2c_params* p, d2c_seq_state* seqs, int32_t batch, void* stream) {
  if (!c) return D2C_EINVAL;
  int rc = check_params(c, p);
  if (rc) return rc;
  if (!seqs || batch <= 0 || batch > c->counts_host_cap) return fail(c, D2C_EINVAL, "bad batch");
  const d2c_dims& D = c->dims;
  for (int b = 0; b < batch; ++b) {
    const d2c_seq_state& s = seqs[b];
    if (!s.tokens || !s.is_masked || !s.k_cache || !s.v_cache || !s.conf || !s.pred || !s.s_idx || !s.s_rows ||
        !s.influence || !s.mstar || !s.u_set || !s.decode_idx || !s.counts)
      return fail(c, D2C_EINVAL, "null buffer in sequence state");
    if (s.L <= 0 || s.L > D.max_seq) return fail(c, D2C_ESHAPE, "L outside (0, max_seq]");
    if (s.n_s < 0 || s.n_s > s.L || s.n_rows < 0 || s.n_rows > s.n_s) return fail(c, D2C_EINVAL, "bad set sizes");
  }
  hipStream_t st = (hipStream_t)stream;
  hipStream_t side = c->tun.side_stream ? c->side : st;
  const int dt = D.dtype, d = D.d_model;
  const size_t ts = tsize(c), cache_layer = (size_t)d_kv(c) * ts;
  const int roll_layers = p->rollout_layers > 0 ? std::min(p->rollout_layers, D.n_layers) : D.n_layers;
  const size_t abar_stride = (size_t)D.max_seq * D.max_seq;
  auto abar_slot = [&](int slot, int layer) { return c->abar_all + ((size_t)slot * D.n_layers + layer) * abar_stride; };
  auto probs_slot = [&](int slot, int layer) {
    return c->probs_all + ((size_t)slot * D.n_layers + layer) * c->probs_elems;
  };
  // sequences are taken in groups of up to max_batch; the rows of a group are projected together
  std::vector<int> group;                       // indices into seqs
  std::vector<Seg> segs;
  for (int b0 = 0; b0 < batch;) {
    group.clear();
    int M = 0;
    while (b0 < batch && (int)group.size() < c->max_batch) {
      d2c_seq_state& s = seqs[b0];
      if (s.n_masked == 0) {
        c->counts_host[(size_t)b0 * D2C_N_COUNTS + D2C_CNT_S] = -1;      // finished: skipped
      } else {
        group.push_back(b0);
        M += s.n_s;
      }
      ++b0;
    }
    if (group.empty()) continue;
    const int n_seg = (int)group.size();
    segs.assign(n_seg, Seg{});
    for (int i = 0, off = 0; i < n_seg; ++i) {
      const d2c_seq_state& s = seqs[group[i]];
      segs[i].idx = s.s_idx;
      segs[i].m = s.n_s;
      segs[i].off = off;
      segs[i].L = s.L;
      off += s.n_s;
    }
    if (M > 0) {
      for (int i = 0; i < n_seg; ++i) {
        const d2c_seq_state& s = seqs[group[i]];
        if (segs[i].m > 0)
          D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
                    launch_embed_norm(dt, c->tok_emb, s.tokens, s.s_idx, segs[i].m, d, c->attn_norm[0], D.rms_eps,
                                      c->hidden + (size_t)segs[i].off * d,
                                      (char*)c->a_norm + (size_t)segs[i].off * d * ts, st));
      }
      for (int l = 0; l < D.n_layers; ++l) {
        const bool in_rollout = l < roll_layers;     // later layers skip the head average altogether
        for (int i = 0; i < n_seg; ++i) {
          const d2c_seq_state& s = seqs[group[i]];
          segs[i].k_cache = (char*)s.k_cache + (size_t)l * s.L * cache_layer;
          segs[i].v_cache = (char*)s.v_cache + (size_t)l * s.L * cache_layer;
          // few rows: the attention launch writes the per-head rows itself and the head means of all layers
          // are taken in one launch after the last layer; otherwise a second pass per layer on the side stream
          const bool emits = attention_fwd_emits_probs(c->tun, dt, segs[i].m, s.L);
          segs[i].probs = in_rollout && emits ? probs_slot(i, l) : nullptr;
          segs[i].abar = in_rollout && !emits ? abar_slot(i, l) : nullptr;
          segs[i].roll_in = nullptr;               // no rollout block here: Eq. 9 comes from the chain below
          segs[i].roll_out = nullptr;
        }
        rc = layer_impl(c, l, c->hidden, segs.data(), n_seg, M, true,
                        l + 1 < D.n_layers ? c->attn_norm[l + 1] : nullptr, st, side, l == roll_layers - 1);
        if (rc) return rc;
      }
      if (side != st) D2C_HIP(c, hipStreamWaitEvent(side, c->fwd_done[roll_layers - 1], 0));
    }
    // Eq. 9 behind the last head average: v = ones, then the layers in reverse order.  On the second stream
    // (if that is on) it runs beside the last layer's FFN, the LM head and Eq. 1.
    for (int i = 0; i < n_seg; ++i) {
      d2c_seq_state& s = seqs[group[i]];
      if (attention_fwd_emits_probs(c->tun, dt, segs[i].m, s.L))
        D2C_TIMED(c, side, D2C_PROF_ATTN_AVG, 0.0,
                  launch_head_mean(probs_slot(i, 0), c->probs_elems, abar_slot(i, 0), abar_stride, roll_layers,
                                   D.n_heads, segs[i].m, s.L, side));
    }
    {
      // the chains of as many sequences as fit the scratch buffers together (sized for one sequence with
      // every row selected) share their three launches
      const size_t Lm = (size_t)D.max_seq;
      std::vector<ChainCall> chain;
      size_t sum_m = 0, sum_mm = 0;
      auto flush_chain = [&]() -> int {
        if (chain.empty()) return D2C_OK;
        D2C_TIMED(c, side, D2C_PROF_ROLLOUT, 0.0,
                  launch_influence_chain(chain.data(), (int)chain.size(), abar_stride, roll_layers, c->chain_u,
                                         c->chain_g, side));
        chain.clear();
        sum_m = sum_mm = 0;
        return D2C_OK;
      };
      for (int i = 0; i < n_seg; ++i) {
        d2c_seq_state& s = seqs[group[i]];
        const size_t m = (size_t)segs[i].m;
        if (!chain.empty() && ((int)chain.size() == chain_max_batch() || sum_m + m > Lm || sum_mm + m * m > Lm * Lm) &&
            (rc = flush_chain()))
          return rc;
        chain.push_back(ChainCall{abar_slot(i, 0), s.s_idx, segs[i].m, s.L, s.influence});
        sum_m += m;
        sum_mm += m * m;
      }
      if ((rc = flush_chain())) return rc;
    }
    if (side != st) D2C_HIP(c, hipEventRecord(c->side_done, side));
    for (int i = 0; i < n_seg; ++i) {
      d2c_seq_state& s = seqs[group[i]];
      const float* hid = c->hidden + (size_t)segs[i].off * d;
      if (segs[i].m > 0 && s.hidden_out)
        D2C_HIP(c, hipMemcpyAsync(s.hidden_out, hid, (size_t)segs[i].m * d * 4, hipMemcpyDeviceToDevice, st));
    }
    // Eq. 1 on the rows of S_t that are still masked: the masked rows of the whole group go through the
    // LM head together, head_rows rows at a time; a piece = rows [r0, r0 + nr) of one sequence's list
    struct Piece { int seg, r0, nr, at; };
    std::vector<Piece> pieces;
    int fill = 0;
    auto flush = [&]() -> int {
      if (fill == 0) return D2C_OK;
      GemmPlan pl;
      size_t stride;
      int rc2 = project(c, c->head_a, d, c->lm_head, fill, D.vocab, d, &pl, &stride, st, true, c->logits);
      if (rc2) return rc2;
      for (const Piece& pc : pieces) {
        d2c_seq_state& s = seqs[group[pc.seg]];
        const float* lg = c->logits + (size_t)pc.at * D.vocab;
        D2C_TIMED(c, st, D2C_PROF_SELECT, 0.0,
                  launch_confidence(lg, s.s_rows + pc.r0, s.s_idx, pc.nr, D.vocab, s.conf, s.pred, c->conf_part, st));
        if (s.logits_out)
          D2C_HIP(c, hipMemcpyAsync(s.logits_out + (size_t)pc.r0 * D.vocab, lg, (size_t)pc.nr * D.vocab * 4,
                                    hipMemcpyDeviceToDevice, st));
      }
      pieces.clear();
      fill = 0;
      return D2C_OK;
    };
    for (int i = 0; i < n_seg; ++i) {
      const d2c_seq_state& s = seqs[group[i]];
      for (int r0 = 0; r0 < s.n_rows;) {
        const int nr = std::min(c->head_rows - fill, s.n_rows - r0);
        D2C_TIMED(c, st, D2C_PROF_ROWWISE, 0.0,
                  launch_gather_norm(dt, c->hidden + (size_t)segs[i].off * d, s.s_rows + r0, nr, d, c->final_norm,
                                     D.rms_eps, (char*)c->head_a + (size_t)fill * d * ts, st));
        pieces.push_back(Piece{i, r0, nr, fill});
        fill += nr;
        r0 += nr;
        if (fill == c->head_rows && (rc = flush())) return rc;
      }
    }
    if ((rc = flush())) return rc;
    // join: the selection is the first consumer of the influence scores, so the chain also runs beside the
    // LM head and Eq. 1
    if (side != st) D2C_HIP(c, hipStreamWaitEvent(st, c->side_done, 0));
    // the selections of the group's sequences share launches (one workgroup per sequence)
    std::vector<SelectArgs> sel;
    for (int i = 0; i < n_seg; ++i) {
      d2c_seq_state& s = seqs[group[i]];
      sel.push_back(SelectArgs{p->sigma, p->k, p->p, p->block_len, p->n_unmask, p->cand_mode, p->threshold, p->conf_decode,
                               s.tokens, s.is_masked, s.L,
                               s.prompt_len, s.conf, s.pred, s.influence, s.mstar, s.u_set, s.decode_idx, s.s_idx, s.s_rows,
                               s.counts, s.score});
      if ((int)sel.size() == select_max_batch() || i + 1 == n_seg) {
        D2C_TIMED(c, st, D2C_PROF_SELECT, 0.0, launch_select(sel.data(), (int)sel.size(), st));
        sel.clear();
      }
    }
    for (int i = 0; i < n_seg; ++i) {
      d2c_seq_state& s = seqs[group[i]];
      D2C_HIP(c, hipMemcpyAsync(c->counts_host + (size_t)group[i] * D2C_N_COUNTS, s.counts,
                                sizeof(int32_t) * D2C_N_COUNTS, hipMemcpyDeviceToHost, st));
    }
  }
  D2C_HIP(c, hipStreamSynchronize(st));
  for (int b = 0; b < batch; ++b) {
    const int32_t* ch = c->counts_host + (size_t)b * D2C_N_COUNTS;
    if (ch[D2C_CNT_S] < 0) continue;
    seqs[b].n_s = ch[D2C_CNT_S];
    seqs[b].n_rows = ch[D2C_CNT_NEXT_ROWS];
    seqs[b].n_masked = ch[D2C_CNT_MASKED];
    seqs[b].step += 1;
  }
  return D2C_OK;
}

}  // extern "C"
