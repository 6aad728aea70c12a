"""CPU oracle for the d2Cache selective-refresh decoding step of a diffusion LLM.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 numpy transcription
of what the paper's method computes.  It shares no code with the HIP library
and must never be imported by the product path: only the tests, the smoke
check and the benchmark's cpu_baseline leg call it.

What follows the paper, and where:
  * the denoising loop, predictions and confidences       -- Sec. 3.1, Eq. 1, Eq. 2
  * certainty density D(i) and stage-1 top-k               -- Sec. 4.1, Eq. 3, Eq. 4
  * partial forward over the rows M* u U                   -- Sec. 4.2, Eq. 5
  * head-averaged attention, expansion, rollout, influence -- Sec. 4.2, Eq. 6-9
  * stage-2 selection by cumulative mass p                 -- Sec. 4.2, last paragraph
The transformer block itself (RMSNorm, rotate-half RoPE, MHA/GQA without a
causal mask, SwiGLU) is not described by the paper, which treats the dLLM as a
given; it is the LLaDA / Dream (Qwen2.5) geometry named in Sec. 5.1.

Readings taken where the paper is silent (each one is a documented choice that
the HIP path takes too):
  R1  F in Eq. 1 is the identity on the maximum softmax probability.
  R2  every arg-max / top-k / sort tie goes to the lowest index.
  R3  M* and the decode set I_t are both drawn from M_t (before unmasking).
  R4  stage-2 candidates are the known tokens {j not in M_t}; cand_mode=1 gives
      the literal alternative {0..L-1} \\ M*.
  R5  a masked token outside this step's forward keeps its cached confidence.
  R6  the "cumulative probability" is c_j normalised over the candidate set.
  R7  a layer writes its new K/V rows into the cache before attending.
  R8  "exceeds p" is strict; if no prefix exceeds, all candidates are taken.
  R9  C^(0) = I at every step: the rollout does not persist across steps.
  R10 selections are taken on float32 score arrays: top-k on (score, index)
      keys, top-p on the fixed-point masses floor(c_j * 2^32) with threshold
      floor(double(p) * double(sum)).
  R11 with block-wise semi-autoregressive decoding the stage-1 and decode
      candidates are the masked tokens of the leftmost unfinished block.
  R15 parallel decoding (appendix, "parallel decoding settings", threshold 0.9):
      besides the n_unmask best-scored candidates, every candidate whose
      confidence s^i exceeds the threshold is unmasked in the same step; the
      threshold is taken on s^i (a probability), not on D(i) s^i.
  R16 confidence-based decoding (the `Conf` rows of the decoding-scheme table):
      the decode set ranks candidates by s^i alone; M* still uses D(i) s^i.
  R17 every token unmasked at step t is fed again at t+1: S_{t+1} = M* u I_t u U
      (equal to M* u U whenever I_t is inside M*, i.e. without R15/R16).
  R18 lightweight rollout (appendix, "lightweight variants of attention
      rollout"): only the first r layers' A-bar enter Eq. 6-8.
  R19 blocks are counted from the end of the prompt by floor division; a masked
      position left of prompt_len (legal input, never produced by the method)
      falls into a block that is clipped at position 0.

Parity status: every function below is pinned by tests/test_oracle_*.py to
closed forms, invariants, library witnesses or brute force.  Agreement with the
authors' own implementation is "parity unpinned": the paper prints no
intermediate value of any of these quantities.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# Parameters and state
# ----------------------------------------------------------------------------
@dataclass
class Dims:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0


@dataclass
class Params:
    """sigma, k, p of Sec. 4 (defaults of Sec. 5.1), plus the decoding schedule."""
    sigma: float = 10.0
    k: int = 32
    p: float = 0.1
    block_len: int = 32
    n_unmask: int = 1
    cand_mode: int = 0
    threshold: float = 0.0        # > 0: parallel decoding by confidence threshold (R15)
    conf_decode: int = 0          # 1: decode by confidence alone (R16)
    rollout_layers: int = 0       # r > 0: rollout over the first r layers only (R18)


@dataclass
class SeqState:
    """Everything one sequence carries from step to step."""
    y: np.ndarray                 # [L] token ids
    is_masked: np.ndarray         # [L] bool, the set M_t
    prompt_len: int
    k_cache: np.ndarray           # [N, L, d_kv] fp64
    v_cache: np.ndarray           # [N, L, d_kv] fp64
    conf: np.ndarray              # [L] float32, s^i of Eq. 1 (cached, R5)
    pred: np.ndarray              # [L] int32, x-hat^i of Eq. 1 (cached, R5)
    S: np.ndarray                 # [m] int32 ascending: rows of the next forward
    trace: Dict = field(default_factory=dict)   # last step's intermediates


# ----------------------------------------------------------------------------
# Transformer block pieces (geometry of Sec. 5.1's models)
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate-half rotary embedding.  x: [rows, heads, d_h]; pos: absolute positions."""
    x = np.asarray(x, F64)
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = np.asarray(theta, F64) ** (-np.arange(half, dtype=F64) / half)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def softmax_rows(z: np.ndarray) -> np.ndarray:
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def selective_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                        n_heads: int, n_kv_heads: int, head_dim: int
                        ) -> Tuple[np.ndarray, np.ndarray]:
    """Attention of the selected query rows against ALL L cached keys, no mask
    (A^(l) in R^{H x |y*| x L}, Sec. 4.2), and its average over the H query
    heads, A-bar^(l).  q: [m, H*d_h]; caches: [L, H_kv*d_h]."""
    m, L = q.shape[0], k_cache.shape[0]
    q = np.asarray(q, F64).reshape(m, n_heads, head_dim)
    K = np.asarray(k_cache, F64).reshape(L, n_kv_heads, head_dim)
    V = np.asarray(v_cache, F64).reshape(L, n_kv_heads, head_dim)
    out = np.zeros((m, n_heads, head_dim), F64)
    abar = np.zeros((m, L), F64)
    group = n_heads // n_kv_heads
    for h in range(n_heads):
        g = h // group
        A = softmax_rows(q[:, h, :] @ K[:, g, :].T / np.sqrt(F64(head_dim)))
        out[:, h, :] = A @ V[:, g, :]
        abar += A
    abar /= n_heads
    return out.reshape(m, n_heads * head_dim), abar


def refresh_layer(dims: Dims, w: Dict[str, np.ndarray], h: np.ndarray, S: np.ndarray,
                  k_cache: np.ndarray, v_cache: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """One block on the compact rows h = hidden[S] (Eq. 5): the rows' new K/V
    replace cache rows S (reading R7), the other cache rows are reused as they
    are.  Returns the new hidden rows and A-bar^(l) [m, L].  Caches change in place."""
    m = len(S)
    H, Hkv, dh = dims.n_heads, dims.n_kv_heads, dims.head_dim
    dq, dkv = H * dh, Hkv * dh
    a = rmsnorm(h, w["attn_norm"], dims.rms_eps)
    qkv = a @ np.asarray(w["wqkv"], F64).T
    if w.get("bqkv") is not None:
        qkv = qkv + np.asarray(w["bqkv"], F64)
    q, k, v = qkv[:, :dq], qkv[:, dq:dq + dkv], qkv[:, dq + dkv:]
    q = rope(q.reshape(m, H, dh), S, dims.rope_theta).reshape(m, dq)
    k = rope(k.reshape(m, Hkv, dh), S, dims.rope_theta).reshape(m, dkv)
    k_cache[S] = k
    v_cache[S] = v
    o, abar = selective_attention(q, k_cache, v_cache, H, Hkv, dh)
    h = np.asarray(h, F64) + o @ np.asarray(w["wo"], F64).T
    b = rmsnorm(h, w["ffn_norm"], dims.rms_eps)
    gu = b @ np.asarray(w["w_gate_up"], F64).T
    g, u = gu[:, :dims.d_ffn], gu[:, dims.d_ffn:]
    act = g / (1.0 + np.exp(-g)) * u
    h = h + act @ np.asarray(w["w_down"], F64).T
    return h, abar


def lm_logits(dims: Dims, model: Dict, h_rows: np.ndarray) -> np.ndarray:
    return rmsnorm(h_rows, model["final_norm"], dims.rms_eps) @ np.asarray(model["lm_head"], F64).T


# ----------------------------------------------------------------------------
# Eq. 1: prediction and confidence
# ----------------------------------------------------------------------------
def confidence(logits: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """x-hat = argmax_v p(v), s = p(x-hat) (Eq. 1 with reading R1).  Ties: lowest v."""
    z = np.asarray(logits, F64)
    xhat = np.argmax(z, axis=-1).astype(np.int32)          # first maximum = lowest index
    p = softmax_rows(z)
    s = p[np.arange(z.shape[0]), xhat]
    return s, xhat


# ----------------------------------------------------------------------------
# Eq. 3, Eq. 4: certainty density and stage-1 selection
# ----------------------------------------------------------------------------
def certainty_density(is_masked: np.ndarray, sigma: float) -> np.ndarray:
    """D(i) = sum_j exp(-|i-j|^2 / (2 sigma^2)) [j not in M], for every i (Eq. 3)."""
    L = len(is_masked)
    pos = np.arange(L, dtype=F64)
    phi = np.exp(-((pos[:, None] - pos[None, :]) ** 2) / (2.0 * F64(sigma) ** 2))
    known = (~np.asarray(is_masked, bool)).astype(F64)
    return phi @ known


def top_k_select(score_f32: np.ndarray, cand: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest scores among cand (Eq. 4), ties to the lowest
    index (R2), decided on float32 values (R10).  Returned ascending."""
    cand = np.asarray(cand, np.int64)
    if k <= 0 or len(cand) == 0:
        return np.zeros(0, np.int32)
    sc = np.asarray(score_f32, np.float32)[cand]
    order = np.lexsort((cand, -sc.astype(F64)))             # primary: score desc; then index asc
    return np.sort(cand[order[:k]]).astype(np.int32)


def current_block(is_masked: np.ndarray, prompt_len: int, block_len: int) -> Tuple[int, int]:
    """Leftmost generation block that still holds a masked token (R11).  With
    block_len >= generation length this is the whole response (the NAR setting)."""
    L = len(is_masked)
    masked = np.flatnonzero(np.asarray(is_masked, bool))
    if len(masked) == 0:
        return L, L
    b = (int(masked[0]) - prompt_len) // block_len          # floor: blocks count from the prompt's end both ways
    lo = prompt_len + b * block_len
    return max(0, lo), min(L, lo + block_len)


# ----------------------------------------------------------------------------
# Eq. 6 - Eq. 9: attention rollout over the expanded matrices
# ----------------------------------------------------------------------------
def expand_attention(abar: np.ndarray, S: np.ndarray, L: int) -> np.ndarray:
    """E^(l): rows in S carry A-bar^(l), every other row is the one-hot e_i (Eq. 6)."""
    E = np.eye(L, dtype=F64)
    if len(S):
        E[np.asarray(S, np.int64), :] = np.asarray(abar, F64)
    return E


def transition(E: np.ndarray) -> np.ndarray:
    """W^(l) = (E^(l) + I) with every row divided by its sum (Eq. 7)."""
    W = E + np.eye(E.shape[0], dtype=F64)
    return W / W.sum(axis=1, keepdims=True)


def rollout(abars: Sequence[np.ndarray], S: np.ndarray, L: int) -> np.ndarray:
    """C^(N) with C^(0) = I and C^(l) = W^(l) C^(l-1) (Eq. 8), on the full L x L matrix."""
    C = np.eye(L, dtype=F64)
    for abar in abars:
        C = transition(expand_attention(abar, S, L)) @ C
    return C


def influence(C: np.ndarray) -> np.ndarray:
    """c_j = sum_i C^(N)_ij (Eq. 9)."""
    return C.sum(axis=0)


def top_p_select(c_f32: np.ndarray, cand: np.ndarray, p: float) -> np.ndarray:
    """Smallest set of candidates, taken in descending c_j, whose share of the
    candidates' total mass exceeds p (Sec. 4.2 last paragraph; R2, R6, R8, R10).
    Returned ascending."""
    cand = np.asarray(cand, np.int64)
    if len(cand) == 0:
        return np.zeros(0, np.int32)
    c = np.asarray(c_f32, np.float32)[cand]
    order = np.lexsort((cand, -c.astype(F64)))
    q = [int(np.floor(F64(v) * 4294967296.0)) for v in c[order]]   # fixed point, exact integers
    total = sum(q)
    threshold = int(np.floor(F64(np.float32(p)) * F64(total)))
    take, run = len(cand), 0
    for r, qv in enumerate(q):
        run += qv
        if run > threshold:
            take = r + 1
            break
    return np.sort(cand[order[:take]]).astype(np.int32)


# ----------------------------------------------------------------------------
# One decoding step and the generation loop (Sec. 3.1 + Sec. 4)
# ----------------------------------------------------------------------------
def new_state(dims: Dims, y0: np.ndarray, is_masked0: np.ndarray, prompt_len: int) -> SeqState:
    L = len(y0)
    dkv = dims.n_kv_heads * dims.head_dim
    return SeqState(
        y=np.array(y0, np.int32), is_masked=np.array(is_masked0, bool), prompt_len=prompt_len,
        k_cache=np.zeros((dims.n_layers, L, dkv), F64), v_cache=np.zeros((dims.n_layers, L, dkv), F64),
        conf=np.zeros(L, np.float32), pred=np.zeros(L, np.int32),
        S=np.arange(L, dtype=np.int32))                     # step 0 feeds the whole y_0


def forward_rows(dims: Dims, model: Dict, st: SeqState, S: np.ndarray
                 ) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Partial forward over rows S (Eq. 5); returns final hidden rows and all A-bar^(l)."""
    h = np.asarray(model["tok_emb"], F64)[st.y[S]]
    abars = []
    for l in range(dims.n_layers):
        h, abar = refresh_layer(dims, model["layers"][l], h, S, st.k_cache[l], st.v_cache[l])
        abars.append(abar)
    return h, abars


def select(params: Params, is_masked: np.ndarray, prompt_len: int, conf: np.ndarray,
           c: np.ndarray) -> Dict[str, np.ndarray]:
    """Two-stage selection plus the decode set, from cached confidences and the
    influence scores.  Returns D, score, M*, I_t, U and S_{t+1} = sort(M* u I_t u U)."""
    L = len(is_masked)
    is_masked = np.asarray(is_masked, bool)
    D = certainty_density(is_masked, params.sigma)
    score = (D * np.asarray(conf, F64)).astype(np.float32)
    lo, hi = current_block(is_masked, prompt_len, params.block_len)
    cand1 = np.array([i for i in range(lo, hi) if is_masked[i]], np.int64)
    mstar = top_k_select(score, cand1, params.k)
    conf32 = np.asarray(conf, np.float32)
    decode = top_k_select(conf32 if params.conf_decode else score, cand1, params.n_unmask)
    if params.threshold > 0:
        sure = [i for i in cand1 if conf32[i] > np.float32(params.threshold)]
        decode = np.union1d(decode, np.array(sure, np.int32)).astype(np.int32)
    if params.cand_mode == 0:
        cand2 = np.flatnonzero(~is_masked)
    else:
        cand2 = np.setdiff1d(np.arange(L), mstar)
    u = top_p_select(np.asarray(c, np.float32), cand2, params.p)
    s_next = np.union1d(np.union1d(mstar, decode), u).astype(np.int32)
    return {"D": D, "score": score, "mstar": mstar, "decode": decode, "u": u, "s_next": s_next,
            "block": (lo, hi)}


def d2cache_step(dims: Dims, model: Dict, params: Params, st: SeqState) -> None:
    """One denoising step: forward over S_t, rollout, Eq. 1 on the masked rows of
    S_t, both selections, unmasking (Eq. 2).  Updates st in place; st.trace keeps
    the intermediates for the tests."""
    L = len(st.y)
    S = np.asarray(st.S, np.int64)
    h, abars = forward_rows(dims, model, st, S)
    r = params.rollout_layers
    C = rollout(abars[:r] if r > 0 else abars, S, L)
    c = influence(C)
    rows = np.array([r for r, i in enumerate(S) if st.is_masked[i]], np.int64)
    logits = np.zeros((0, dims.vocab), F64)
    if len(rows):
        logits = lm_logits(dims, model, h[rows])
        s, xhat = confidence(logits)
        st.conf[S[rows]] = s.astype(np.float32)
        st.pred[S[rows]] = xhat
    sel = select(params, st.is_masked, st.prompt_len, st.conf, c.astype(np.float32))
    dec = sel["decode"]
    st.y[dec] = st.pred[dec]
    st.is_masked[dec] = False
    st.trace = dict(sel, S=S.astype(np.int32), hidden=h, abars=abars, C=C, c=c,
                    logit_rows=S[rows].astype(np.int32), logits=logits)
    st.S = sel["s_next"]


def generate(dims: Dims, model: Dict, params: Params, y0: np.ndarray, is_masked0: np.ndarray,
             prompt_len: int, max_steps: Optional[int] = None, on_step=None) -> SeqState:
    """Run the loop of Sec. 3.1 until M = {} (or max_steps)."""
    st = new_state(dims, y0, is_masked0, prompt_len)
    t = 0
    while st.is_masked.any() and (max_steps is None or t < max_steps):
        d2cache_step(dims, model, params, st)
        if on_step is not None:
            on_step(t, st)
        t += 1
    return st


# ----------------------------------------------------------------------------
# Full recomputation (the paper's "Vanilla": every step recomputes all rows).
# Written separately from refresh_layer, position by position, so that the
# "select everything == full recomputation" check compares two codes.
# ----------------------------------------------------------------------------
def full_forward(dims: Dims, model: Dict, y: np.ndarray) -> Dict[str, np.ndarray]:
    L = len(y)
    H, Hkv, dh, F = dims.n_heads, dims.n_kv_heads, dims.head_dim, dims.d_ffn
    x = np.asarray(model["tok_emb"], F64)[np.asarray(y, np.int64)].copy()
    half = dh // 2
    freqs = np.array([dims.rope_theta ** (-(i / half)) for i in range(half)], F64)
    keys, values, attn_mean = [], [], []
    for w in model["layers"]:
        Wqkv, Wo = np.asarray(w["wqkv"], F64), np.asarray(w["wo"], F64)
        Wgu, Wd = np.asarray(w["w_gate_up"], F64), np.asarray(w["w_down"], F64)
        Q = np.zeros((L, H, dh)); K = np.zeros((L, Hkv, dh)); V = np.zeros((L, Hkv, dh))
        for t in range(L):
            xn = x[t] / np.sqrt(np.dot(x[t], x[t]) / len(x[t]) + dims.rms_eps) * w["attn_norm"]
            proj = Wqkv @ xn
            if w.get("bqkv") is not None:
                proj = proj + w["bqkv"]
            qt = proj[:H * dh].reshape(H, dh)
            kt = proj[H * dh:H * dh + Hkv * dh].reshape(Hkv, dh)
            V[t] = proj[H * dh + Hkv * dh:].reshape(Hkv, dh)
            cs, sn = np.cos(t * freqs), np.sin(t * freqs)
            for src, dst in ((qt, Q), (kt, K)):
                dst[t, :, :half] = src[:, :half] * cs - src[:, half:] * sn
                dst[t, :, half:] = src[:, half:] * cs + src[:, :half] * sn
        att_out = np.zeros((L, H * dh))
        amean = np.zeros((L, L))
        for hh in range(H):
            g = hh * Hkv // H
            logits = np.einsum("td,sd->ts", Q[:, hh], K[:, g]) / np.sqrt(dh)
            logits -= logits.max(axis=1, keepdims=True)
            P = np.exp(logits)
            P /= P.sum(axis=1, keepdims=True)
            att_out[:, hh * dh:(hh + 1) * dh] = P @ V[:, g]
            amean += P / H
        x = x + att_out @ Wo.T
        for t in range(L):
            xn = x[t] / np.sqrt(np.dot(x[t], x[t]) / len(x[t]) + dims.rms_eps) * w["ffn_norm"]
            gu = Wgu @ xn
            g_, u_ = gu[:F], gu[F:]
            x[t] = x[t] + Wd @ (g_ / (1.0 + np.exp(-g_)) * u_)
        keys.append(K.reshape(L, Hkv * dh)); values.append(V.reshape(L, Hkv * dh))
        attn_mean.append(amean)
    xn = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + dims.rms_eps) * model["final_norm"]
    return {"hidden": x, "logits": xn @ np.asarray(model["lm_head"], F64).T,
            "k": np.stack(keys), "v": np.stack(values), "attn_mean": attn_mean}
