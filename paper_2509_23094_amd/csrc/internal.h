// Host-side launch interface between the C ABI layer and the kernel files.
// Every launcher checks its own shape assumptions and returns hipError_t.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace d2c {

enum DType { kF32 = 0, kBF16 = 1 };

inline size_t dtype_size(int dt) { return dt == kBF16 ? 2 : 4; }

// Launch-shape tunables.  Every context holds its own copy (defaults chosen by measurement); the tooling
// calls d2c_init_tuned / d2c_ctx_set_tunable change them per context.
struct Tunables {
  int gemm_target_wgs = 384;   // aim for at least this many groups of 4 waves per GEMM
  int gemm_max_splits = 8;
  int gemm_wide_min_rows = 257; // the wide instantiation from this many rows on (3 row chunks)
  int gemm_tall_chunk = 1;      // 129-192 bf16 rows as ONE row chunk of 10 or 12 row tiles
  int gemm_wide_tiles = 1;     // more than 128 rows in bf16: 128 x 64 outputs per wave, 4 waves per workgroup
  int gemm_wide_mt = 0;        // row tiles per workgroup of the wide instantiation: 6, 7, 8; 0 = by shape
  int gemm_nt_big_n = 1 << 30; // N above this uses two column tiles per wave even for few rows (measured slower);
                               // more than 128 rows always do
  int gemm_waves = 0;          // waves per workgroup sharing one activation chunk in LDS: 4, 6, 8, 10; 0 = by shape
  bool gemm_preshuffle = true; // d2c_init keeps pre-tiled copies of the projection matrices (costs their size again)
  int gemm_rot = 0;            // start chunk of a workgroup's k walk = (column block * this) % chunks
  int attn_tiled_min_m = 96;   // bf16 attention: from this many query rows on, the LDS-tiled kernels
  int attn_max_splits = 8;     // key-range splits of one attention launch (1..8)
  int attn_qt = 0;             // 16-row query tiles per wave in the tiled forward kernel: 1, 2; 0 = by m
  int attn_waves = 0;          // waves per workgroup of the tiled forward kernel: 4, 8; 0 = by m
  int attn_target_wgs = 256;   // split the key range until the forward grid has this many workgroups
  bool side_stream = false;    // d2c_step: head average + rollout on a second stream (measured slower: with two
                               // queues in use every launch of the step takes longer than the overlap saves)
};
// name -> field; false for an unknown name
bool set_tunable(Tunables& t, const char* name, int value);

// ---- GEMM on a ragged handful of rows: P[s] = A[m,K] * W[N,K]^T over the k-range of split s
struct GemmPlan {
  int mt;        // 16-row tiles per workgroup (1..8)
  int nt;        // 16-column tiles per wave (1 or 2)
  int waves;     // waves per workgroup (4, 8 or 16), each owning 16*nt output columns
  int splits;    // k splits (partials to be summed by the consumer)
  int k_per_split;
  int row_chunks;
  int rot;       // multiplier of the per-workgroup start-chunk rotation (0 = none)
};
GemmPlan plan_gemm(const Tunables& t, int dtype, int m, int N, int K, bool single_split = false);
// P must hold plan.splits * split_stride floats; split_stride >= m * ldp.
// pre = W is a pre-tiled copy made by launch_preshuffle (then ldw = 256-byte chunks per row).
hipError_t launch_gemm(int dtype, const GemmPlan& plan, const void* A, int lda, const void* W, int ldw,
                       float* P, int ldp, size_t split_stride, int m, int N, int K, hipStream_t st,
                       bool pre = false);
// Pre-tiled weight copy: 16-row x 256-byte blocks, each stored as the 4 x 1 KB wave loads of the
// projection kernel ([tile][chunk][step][lane][16 B]); rows and row tails are zero-padded.
size_t preshuffled_bytes(int N, int K, int dtype);
// interleave_half = F > 0 (N = 2F, F % 16 == 0): 16-row tiles of the two halves alternate (gate, up, gate, ..).
hipError_t launch_preshuffle(int dtype, const void* W, int ldw, int N, int K, void* dst, hipStream_t st,
                             int interleave_half = 0);
// act[m, F] = T(silu(g) * u) with [g | u] = A W^T, W a pre-tiled interleaved copy of [2F, K]; plan: single split
hipError_t launch_gemm_swiglu(int dtype, const GemmPlan& plan, const void* A, int lda, const void* W, int ldw,
                              void* act, int F, int m, int K, hipStream_t st);

// ---- row-wise kernels
// h[r,:] = emb[tokens[idx[r]],:];  a[r,:] = T(rmsnorm(h[r,:]) * gain)
hipError_t launch_embed_norm(int dtype, const void* emb, const int32_t* tokens, const int32_t* idx, int m, int d,
                             const float* gain, float eps, float* h, void* a, hipStream_t st);
// h[r,:] += bias? + sum_s P[s][r,:] (n_splits may be 0);  if a: a[r,:] = T(rmsnorm(h[r,:]) * gain)
hipError_t launch_add_norm(int dtype, float* h, const float* P, int n_splits, size_t split_stride, int ldp, int m,
                           int d, const float* gain, float eps, void* a, hipStream_t st);
// a[i,:] = T(rmsnorm(h[rows[i],:]) * gain)
hipError_t launch_gather_norm(int dtype, const float* h, const int32_t* rows, int n_rows, int d, const float* gain,
                              float eps, void* a, hipStream_t st);
// split sums of the QKV projection (+bias), RoPE on q and k at the rows' positions; q -> q_out[r,:],
// k -> k_cache[pos,:], v -> v_cache[pos,:].  The compact rows are the concatenation of up to rope_max_batch
// sequences' slices (off = first row of the slice; slices consecutive and non-empty), each with its own
// index set (pos = idx[r - off]) and caches.
struct RopeCall {
  const int32_t* idx;
  void *k_cache, *v_cache;
  int off, m;
};
int rope_max_batch();
hipError_t launch_qkv_rope_scatter(int dtype, const float* P, int n_splits, size_t split_stride, int ldp,
                                   const float* bias, const RopeCall* calls, int n_calls, int n_heads, int n_kv_heads,
                                   int head_dim, const float* rope_cos, const float* rope_sin, void* q_out,
                                   hipStream_t st);
// act[r,f] = T(silu(g) * u), g/u = split sums of columns f and F+f
hipError_t launch_swiglu(int dtype, const float* P, int n_splits, size_t split_stride, int ldp, int m, int F,
                         void* act, hipStream_t st);
// cache_a[idx[r],:] = rows_a[r,:] and, when rows_b is given, cache_b[idx[r],:] = rows_b[r,:].
// Pointers and width*sizeof(T) must be multiples of 16 bytes for the wide path (else element copies).
hipError_t launch_scatter_rows(int dtype, const void* rows_a, void* cache_a, const void* rows_b, void* cache_b,
                               const int32_t* idx, int m, int width, hipStream_t st);
hipError_t launch_copy_f32(float* dst, const float* src, size_t n, hipStream_t st);
// dst[i] = sum_s P[s*split_stride + i], i < n
hipError_t launch_sum_splits(float* dst, const float* P, int n_splits, size_t split_stride, size_t n, hipStream_t st);
// cos/sin table [max_pos, head_dim/2], angles evaluated in fp64
hipError_t launch_rope_table(float* cos_t, float* sin_t, int max_pos, int head_dim, float theta, hipStream_t st);

// ---- attention of m query rows against all L cached keys, no mask
// Two kernel families.  Few query rows (fp32, or bf16 below attn_tiled_min_m rows): a forward launch and, for
// the head average, either per-head probability rows written by the forward launch itself (probs, see
// attention_fwd_emits_probs) or a second launch (launch_attention_avg) that needs the forward's lse.  Many
// rows in bf16 (attention_is_tiled: attn_tiled_min_m rows, or 48 already when the key range is too long
// for the probability rows): K/V blocks staged through LDS, key range split over workgroups; the
// forward launch also leaves what the head average needs, and one finishing launch merges the splits and
// writes the average, so tiled_avg is given to launch_attention_fwd itself.
// fwd: out T [m, H*dh] and the log-sum-exp per (head, row), lse float [H, m]
// scratch: attention_scratch_floats(...) floats, may be null for fp32
bool attention_is_tiled(const Tunables& t, int dtype, int m, int L);
size_t attention_scratch_floats(const Tunables& t, int dtype, int max_m, int max_L, int n_heads, int head_dim);
// probs (optional, only where attention_fwd_emits_probs): bf16 [H, m, L], the normalised attention rows of
// every head, written by the same launch; launch_head_mean turns them into the head average.
bool attention_fwd_emits_probs(const Tunables& t, int dtype, int m, int L);
size_t attention_probs_elems(int dtype, int n_heads, int max_L);       // bf16 elements one (layer, sequence) needs
// tiled_avg: float [m, L] or null; only read where attention_is_tiled (elsewhere it must be null)
hipError_t launch_attention_fwd(const Tunables& t, int dtype, const void* q, const void* k_cache, const void* v_cache, int m, int L,
                                int n_heads, int n_kv_heads, int head_dim, void* out, float* lse, float* scratch,
                                size_t scratch_floats, hipStream_t st, void* probs = nullptr,
                                float* tiled_avg = nullptr);
// abar[l] (at abar + l * abar_layer_stride, [m, L]) = mean over heads of probs[l] (at probs + l * stride, [H, m, L])
hipError_t launch_head_mean(const void* probs, size_t probs_layer_stride, float* abar, size_t abar_layer_stride,
                            int n_layers, int n_heads, int m, int L, hipStream_t st);
// the second launch of the few-row kernels: attn_avg float [m, L] = mean over heads of
// exp(q k / sqrt(dh) - lse); needs fwd's lse.  Not for attention_is_tiled shapes.
hipError_t launch_attention_avg(const Tunables& t, int dtype, const void* q, const void* k_cache, const float* lse, int m, int L,
                                int n_heads, int n_kv_heads, int head_dim, float* attn_avg, hipStream_t st);

// the bf16 kernels for many query rows: forward over a split key range, then one launch that merges the
// splits and (attn_avg != null) writes the head average.  Several sequences (up to attention_tiled_max_batch)
// share the two launches: together they fill the chip with fewer key splits, i.e. fewer partials to merge.
// The scratch is cut into one piece per sequence: it must hold the sum of their needs.
struct TiledCall {
  const void *q, *k_cache, *v_cache;
  int m, L;
  void* out;          // T [m, H*dh]
  float* lse;         // [H, m]
  float* attn_avg;    // [m, L] or null
};
int attention_tiled_max_batch();
size_t attention_tiled_scratch_floats(const Tunables& t, int max_m, int max_L, int n_heads, int head_dim);
hipError_t launch_attention_tiled(const Tunables& t, const TiledCall* calls, int n_calls, int n_heads, int n_kv_heads,
                                  int head_dim, float* scratch, size_t scratch_floats, hipStream_t st);

// ---- rollout on the compact block: c_out = (A[:,S] c_in + A[:,notS] + c_in) / 2; first: c_in = one-hot rows
hipError_t launch_rollout(const float* attn_avg, const float* c_in, float* c_out, const int32_t* idx, int m, int L,
                          bool first, hipStream_t st);
hipError_t launch_influence(const float* c_block, const int32_t* idx, int m, int L, float* influence,
                            hipStream_t st);

// ---- Eq. 9 as a row-vector chain: c = 1^T W^(n_layers) ... W^(1) with W^(l) built from abar_l (Eq. 6-7),
// for up to chain_max_batch() independent sequences at once.  abar: layer l of a sequence at abar + l *
// layer_stride, [m, L] floats.  u_scratch: n_layers * (sum of m) floats, g_scratch: n_layers * (sum of m * m)
// floats.  Three launches (the m x m blocks made dense, the sequential m x m part in one workgroup per
// sequence, then all columns in parallel); L <= the selection kernel's limit.
// m == 0 or n_layers == 0: all ones.
struct ChainCall {
  const float* abar;
  const int32_t* idx;
  int m, L;
  float* influence;
};
int chain_max_batch();
hipError_t launch_influence_chain(const ChainCall* calls, int n_calls, size_t layer_stride, int n_layers,
                                  float* u_scratch, float* g_scratch, hipStream_t st);

// ---- selection
// Eq. 1 per logits row; the row's position is via ? via[pos[row]] : pos[row]
// scratch: confidence_scratch_floats(n_rows) floats
size_t confidence_scratch_floats(int n_rows);
hipError_t launch_confidence(const float* logits, const int32_t* pos, const int32_t* via, int n_rows, int vocab,
                             float* conf, int32_t* pred, float* scratch, hipStream_t st);
struct SelectArgs {
  float sigma; int k; float p; int block_len; int n_unmask; int cand_mode; float threshold; int conf_decode;
  int32_t* tokens; uint8_t* is_masked; int L; int prompt_len;
  const float* conf; const int32_t* pred; const float* influence;
  int32_t *mstar, *u_set, *decode_idx, *s_next, *s_rows_next, *counts;
  float* score_out;   // nullable: D(i) * s^i of the stage-1 candidates, 0 elsewhere
};
int select_max_len();
// n independent sequences (n <= select_max_batch), one workgroup each
int select_max_batch();
hipError_t launch_select(const SelectArgs* args, int n, hipStream_t st);
hipError_t launch_seq_reset(const uint8_t* is_masked, int L, int32_t* s_idx, int32_t* s_rows, float* conf,
                            int32_t* pred, int32_t* counts, hipStream_t st);

}  // namespace d2c
