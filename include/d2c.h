/*
 * d2c.h -- C ABI of the MI355X (gfx950) d2Cache selective-refresh decoding step
 * for diffusion LLMs.
 *
 * One denoising step (Sec. 3.1 of the d2Cache paper) has two parts:
 *   1. two-stage token selection (Sec. 4.1, Sec. 4.2): certainty-prior top-k over
 *      the masked tokens, then attention-rollout top-p over the known tokens;
 *   2. a partial forward pass over only the selected rows (Eq. 5): their new
 *      K/V rows replace the cached ones, they attend to the whole cache without
 *      a mask, and the head-averaged attention rows feed the rollout (Eq. 6-8).
 *
 * Conventions for every call
 *   - returns 0 (D2C_OK) or a negative error code; never throws or aborts;
 *     on an argument error nothing has been launched or written;
 *   - every tensor pointer is a DEVICE pointer borrowed for the duration of the
 *     call unless it is marked (host); the caller owns all of them;
 *   - `stream` is a hipStream_t passed as void*; all work is asynchronous on it,
 *     except d2c_step, which ends with one small device-to-host copy and a
 *     stream synchronisation (the next step's launch shapes depend on it);
 *   - activations are row-major [rows, features]; weights are row-major
 *     [out_features, in_features]; index sets are int32, ascending, distinct;
 *   - storage type T is float (D2C_F32) or bfloat16 (D2C_BF16): weights,
 *     embeddings and the K/V cache are T; the residual stream, logits,
 *     attention averages, rollout, confidences and norm gains are float;
 *   - timing, launch-shape tunables and the launch planner are tooling and live in d2c_tools.h;
 *   - a context is not thread-safe: calls that share a d2c_ctx must be issued
 *     from one thread at a time and on one stream at a time (they share the
 *     context's workspace).
 */
#ifndef D2C_H
#define D2C_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define D2C_OK       0
#define D2C_EINVAL  (-1)   /* null pointer, bad index set, bad parameter        */
#define D2C_ENOMEM  (-2)   /* workspace allocation failed                       */
#define D2C_EHIP    (-3)   /* a HIP runtime call failed (see d2c_last_error)    */
#define D2C_ESHAPE  (-4)   /* a size exceeds what the context was created for   */

#define D2C_F32   0
#define D2C_BF16  1

typedef struct d2c_ctx d2c_ctx;   /* opaque; created by d2c_init, freed by d2c_destroy */

/* Geometry of the given dLLM (LLaDA / Dream style block: RMSNorm, rotate-half
 * RoPE, MHA or GQA without causal mask, SwiGLU).  The paper treats the model as
 * given (Sec. 3.1); these are the fields of the two models of Sec. 5.1. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t max_seq;      /* largest sequence length L any later call will use     */
  int32_t dtype;        /* D2C_F32 or D2C_BF16                                    */
  float   rms_eps;
  float   rope_theta;
  int32_t mask_id;      /* id of the [MASK] token (Sec. 3.1)                      */
  int32_t max_batch;    /* sequences whose selected rows one d2c_step projects together
                           (the weights are then streamed once per group, not once per
                           sequence); the row-sized workspace grows with it; 0 = 1     */
} d2c_dims;

/* Borrowed device pointers.  The per-layer members are HOST arrays of n_layers
 * device pointers.  wqkv rows: Q (n_heads*head_dim), then K, then V (each
 * n_kv_heads*head_dim); w_gate_up rows: gate (d_ffn) then up (d_ffn).
 * bqkv may be NULL (no bias) or hold float vectors of length rows(wqkv). */
typedef struct {
  const void*        tok_emb;      /* T [vocab, d_model]                          */
  const float*       final_norm;   /* [d_model]                                   */
  const void*        lm_head;      /* T [vocab, d_model]                          */
  const float* const* attn_norm;   /* (host)[n_layers] -> [d_model]               */
  const void*  const* wqkv;        /* (host)[n_layers] -> T [d_q + 2 d_kv, d_model] */
  const float* const* bqkv;        /* (host)[n_layers] -> [d_q + 2 d_kv], or NULL */
  const void*  const* wo;          /* (host)[n_layers] -> T [d_model, d_q]        */
  const float* const* ffn_norm;    /* (host)[n_layers] -> [d_model]               */
  const void*  const* w_gate_up;   /* (host)[n_layers] -> T [2 d_ffn, d_model]    */
  const void*  const* w_down;      /* (host)[n_layers] -> T [d_model, d_ffn]      */
} d2c_weights;

/* Hyper-parameters of Sec. 4 (defaults of Sec. 5.1: sigma 10, k 32, p 0.1) and
 * the decoding schedule.  block_len >= generation length gives the fully
 * non-autoregressive setting; cand_mode 0 draws stage-2 candidates from the
 * known tokens, 1 from every token outside M*. */
typedef struct {
  float   sigma;
  int32_t k;
  float   p;
  int32_t block_len;
  int32_t n_unmask;
  int32_t cand_mode;
  float   threshold;       /* > 0: parallel decoding -- every stage-1 candidate whose confidence s^i
                              exceeds it is unmasked too (appendix, parallel decoding, 0.9); 0 = off */
  int32_t conf_decode;     /* 1: the decode set ranks by s^i alone (the `Conf` decoding of the
                              decoding-scheme table); M* still ranks by D(i) s^i                   */
  int32_t rollout_layers;  /* r > 0: only the first r layers enter the rollout (appendix,
                              lightweight rollout); 0 = all layers                                  */
} d2c_params;

/* Slots of the `counts` array written by d2c_select. */
enum {
  D2C_CNT_MSTAR = 0,      /* |M*|                                                 */
  D2C_CNT_U = 1,          /* |U|                                                  */
  D2C_CNT_S = 2,          /* |S_{t+1}| = |M* u I_t u U|                           */
  D2C_CNT_DECODE = 3,     /* |I_t|                                                */
  D2C_CNT_NEXT_ROWS = 4,  /* members of S_{t+1} still masked after unmasking      */
  D2C_CNT_MASKED = 5,     /* |M_{t+1}|                                            */
  D2C_CNT_BLOCK_LO = 6,   /* current block [lo, hi)                               */
  D2C_CNT_BLOCK_HI = 7,
  D2C_N_COUNTS = 8
};

/* Per-sequence decoding state: caller-owned device buffers plus host mirrors of
 * the set sizes.  d2c_seq_reset prepares it for step 0. */
typedef struct {
  int32_t* tokens;       /* [L]  y_t, updated in place (Eq. 2)                    */
  uint8_t* is_masked;    /* [L]  1 where i is in M_t                              */
  void*    k_cache;      /* T [n_layers, L, d_kv]                                 */
  void*    v_cache;      /* T [n_layers, L, d_kv]                                 */
  float*   conf;         /* [L]  cached s^i of Eq. 1                              */
  int32_t* pred;         /* [L]  cached x-hat^i of Eq. 1                          */
  int32_t* s_idx;        /* [L]  S_t on entry, S_{t+1} on return (n_s valid)      */
  int32_t* s_rows;       /* [L]  compact rows r of S with s_idx[r] masked (n_rows valid) */
  float*   influence;    /* [L]  out: c_j of this step (Eq. 9)                    */
  int32_t* mstar;        /* [L]  out: M* ascending                                */
  int32_t* u_set;        /* [L]  out: U ascending                                 */
  int32_t* decode_idx;   /* [L]  out: I_t ascending                               */
  int32_t* counts;       /* [D2C_N_COUNTS] out                                    */
  float*   score;        /* nullable: [L] out: D(i)*s^i of the stage-1 candidates, 0 elsewhere */
  float*   hidden_out;   /* nullable: [n_s, d_model] final hidden rows of the step */
  float*   logits_out;   /* nullable: [n_rows, vocab] logits of the step          */
  int32_t  L, prompt_len;
  int32_t  n_s, n_rows, n_masked;   /* (host) sizes of s_idx / s_rows, |M_t|      */
  int32_t  step;                    /* (host) steps taken so far                  */
} d2c_seq_state;

/* Validates dims, records the weight pointers, allocates the workspace (sized
 * by max_seq) and builds the RoPE table.  Uses the current HIP device. */
int d2c_init(const d2c_dims* dims, const d2c_weights* weights, d2c_ctx** out);
int d2c_destroy(d2c_ctx* ctx);
/* Text of the last error of this context (or of d2c_init when ctx is NULL).
 * The pointer stays valid until the next failing call. */
const char* d2c_last_error(const d2c_ctx* ctx);

/* Step-0 state (Sec. 3.1): S_0 = every row, s_rows = the masked rows, conf = 0,
 * counts from is_masked.  tokens / is_masked must already hold y_0 and M_0.
 * Synchronises the stream once to read |M_0|. */
int d2c_seq_reset(d2c_ctx* ctx, d2c_seq_state* seq, void* stream);

/* Two-stage selection (Sec. 4.1 + 4.2) and unmasking (Eq. 2) for one sequence.
 *   logits [n_rows, vocab] float, logit_pos [n_rows]: positions those rows
 *   belong to; Eq. 1 on them refreshes conf/pred at those positions (n_rows may
 *   be 0, then logits may be NULL).
 *   influence [L]: c_j of Eq. 9.
 * Then: D(i) (Eq. 3), score D(i)*conf[i]; M* = top-k (Eq. 4) and I_t = top-n_unmask
 * over the masked tokens of the leftmost unfinished block of block_len
 * generation slots; U = smallest prefix, in descending c_j, of the candidates
 * whose mass exceeds p * (candidates' total) (ties to the lowest index; masses
 * in fixed point floor(c*2^32)); tokens[i] <- pred[i], is_masked[i] <- 0 for
 * i in I_t.  Outputs (ascending): mstar, u_set, decode_idx, s_next = M* u I_t u U,
 * s_rows_next = rows r of s_next whose token is still masked, counts, and (if
 * score_out is not NULL) the float scores D(i)*conf[i] the top-k was taken on,
 * 0 outside the stage-1 candidates.  influence must be finite and >= 0.
 * L <= max_seq. */
int d2c_select(d2c_ctx* ctx, const d2c_params* params,
               const float* logits, const int32_t* logit_pos, int32_t n_rows,
               int32_t* tokens, uint8_t* is_masked, int32_t L, int32_t prompt_len,
               float* conf, int32_t* pred, const float* influence,
               int32_t* mstar, int32_t* u_set, int32_t* decode_idx,
               int32_t* s_next, int32_t* s_rows_next, int32_t* counts, float* score_out,
               void* stream);

/* d2c_select for callers that cannot allocate device memory or hold a context: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error codes as
 * d2c_select, with the vocabulary size passed in place of the context.  The call allocates nothing (no
 * hipMalloc / hipFree, no context, no workspace): the only scratch its kernels need -- Eq. 1's per-chunk
 * (max, argmax, sum) triples -- lives in an array inside the library's device code, 192 KiB per GPU, held
 * until the process ends.  Limits: n_rows <= D2C_STATIC_MAX_ROWS and L <= 4096, else D2C_ESHAPE.
 * Every call on a GPU shares that GPU's one array (nothing in it has to be cleared between calls): calls
 * that overlap in time on one GPU, on any streams, race; issue them one after the other.
 * d2c_last_error(NULL) holds the text of its last error. */
#define D2C_STATIC_MAX_ROWS 256
int d2c_select_static(const d2c_params* params, int32_t vocab,
                      const float* logits, const int32_t* logit_pos, int32_t n_rows,
                      int32_t* tokens, uint8_t* is_masked, int32_t L, int32_t prompt_len,
                      float* conf, int32_t* pred, const float* influence,
                      int32_t* mstar, int32_t* u_set, int32_t* decode_idx,
                      int32_t* s_next, int32_t* s_rows_next, int32_t* counts, float* score_out,
                      void* stream);

/* One transformer block on the m selected rows (Eq. 5).
 *   hidden [m, d_model] float, in/out (compact rows, row r is position idx[r]);
 *   idx (host copy idx_host is validated: ascending, distinct, in [0, L));
 *   k_cache / v_cache: T [L, d_kv] of this layer; rows idx are overwritten with
 *   the rows' new (RoPE'd) K and V BEFORE attention, all other rows are read only;
 *   attn_avg [m, L] float out: mean over the query heads of the softmax rows;
 *   rollout [m, L] float in/out: the block C_S of the rollout matrix (rows
 *   outside S stay one-hot, Eq. 6-8): C_S <- (A[:,S] C_S + A[:,not S] + C_S)/2.
 *   When layer == 0 the incoming rollout is ignored (C^(0) = I).
 *   attn_avg and rollout may both be NULL (no rollout wanted).
 * m == 0 is legal and touches nothing. */
int d2c_refresh_layer(d2c_ctx* ctx, int32_t layer, float* hidden,
                      const int32_t* idx, const int32_t* idx_host, int32_t m,
                      void* k_cache, void* v_cache, int32_t L,
                      float* attn_avg, float* rollout, void* stream);

/* Isolated selective-refresh attention: scatter new_k/new_v (T [m, d_kv], may be
 * NULL to skip the scatter) into cache rows idx, then attention of q (T [m, d_q])
 * against all L cache rows, no mask.  out: T [m, d_q]; attn_avg: float [m, L] or NULL. */
int d2c_attention(d2c_ctx* ctx, const void* q, const int32_t* idx, int32_t m,
                  const void* new_k, const void* new_v, void* k_cache, void* v_cache,
                  int32_t L, void* out, float* attn_avg, void* stream);

/* The projection kernel on its own: out[m, N] (float) = a[m, K] * w[N, K]^T with a and w
 * of storage type T and fp32 accumulation -- the ragged-row, weight-streaming GEMM
 * every projection of the partial forward (Eq. 5) runs through.  K and the row
 * pitches must be multiples of 16 bytes of T; m <= max_seq. */
int d2c_linear(d2c_ctx* ctx, const void* a, const void* w, int32_t m, int32_t N, int32_t K,
               float* out, void* stream);

/* c_j = [j not in S] + sum_i C_S[i, j] (Eq. 9 on the compact block). */
int d2c_influence(d2c_ctx* ctx, const float* rollout, const int32_t* idx, int32_t m,
                  int32_t L, float* influence, void* stream);

/* One whole denoising step for `batch` independent sequences: partial forward
 * over S_t through all layers with rollout, LM head and Eq. 1 on the masked rows
 * of S_t, selection and unmasking; leaves S_{t+1} in the state and refreshes the
 * host mirrors.  A sequence with n_masked == 0 is skipped.  The sequences are independent (own
 * caches, sets, rollout); they are taken in groups of up to max_batch whose rows share the
 * projection launches; the other kernels work on each sequence's own slice (several sequences
 * of a group per launch where the kernel allows it). */
int d2c_step(d2c_ctx* ctx, const d2c_params* params, d2c_seq_state* seqs, int32_t batch,
             void* stream);

/* Bytes of device workspace the context holds. */
int64_t d2c_workspace_bytes(const d2c_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* D2C_H */
