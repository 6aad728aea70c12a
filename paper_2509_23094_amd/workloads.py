"""Seeded synthetic inputs for the d2Cache selective-refresh step.

This module is the only code shared by the CPU oracle's tests and the HIP path.
It holds no arithmetic of the method: it only draws random weights, token ids,
K/V tensors and index sets with the shapes of the two dLLMs the paper runs
(LLaDA-8B and Dream-7B geometry, Sec. 5.1 "Experimental setup") and of the small
test cases.  Every tensor has its own counter-seeded stream, so any subset (one
layer, the LM head only) can be drawn without drawing the rest.

All arrays are numpy float32.  For the bf16 workloads every value is rounded
once to a bf16-representable number, so that both sides start from the same
bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterable, Optional

import numpy as np


@dataclass(frozen=True)
class ModelDims:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # "f32" | "bf16": storage type of weights and K/V
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def mask_id(self) -> int:
        return self.vocab - 1

    @property
    def d_q(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim


@dataclass(frozen=True)
class DecodeSetup:
    prompt_len: int
    gen_len: int
    block_len: int
    n_unmask: int
    k: int
    p: float
    sigma: float = 10.0
    batch: int = 1

    @property
    def seq_len(self) -> int:
        return self.prompt_len + self.gen_len


# The workloads.  C3-C6 use the paper's default hyper-parameters
# (sigma = 10, k = 32, p = 0.1; "Implementation details" in Sec. 5.1).
DIMS = {
    "C1": ModelDims(2, 256, 4, 4, 64, 688, 1024, dtype="f32"),
    "C3": ModelDims(32, 4096, 32, 32, 128, 12288, 126464, dtype="bf16"),
    "C4": ModelDims(28, 3584, 28, 4, 128, 18944, 152064, dtype="bf16"),
}
DIMS["C5"] = DIMS["C3"]
DIMS["C6"] = DIMS["C4"]
SETUP = {
    "C1": DecodeSetup(64, 64, 32, 1, k=8, p=0.9),
    "C3": DecodeSetup(256, 256, 32, 1, k=32, p=0.1),
    "C4": DecodeSetup(512, 256, 32, 1, k=32, p=0.1),
    "C5": DecodeSetup(2048, 1024, 64, 2, k=32, p=0.1, batch=4),
    # long generation at the Dream-7B shape (the long-context table of Appendix: gen 1024, prompts up to ~800)
    "C6": DecodeSetup(800, 1024, 32, 1, k=32, p=0.1),
}


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


_TENSOR_IDS = {
    "tok_emb": 1, "lm_head": 2, "wqkv": 3, "wo": 4, "w_gate_up": 5, "w_down": 6,
    "prompt": 7, "attn_q": 8, "attn_k": 9, "attn_v": 10, "attn_newk": 11,
    "attn_newv": 12, "attn_idx": 13, "hidden": 14, "logits": 15, "scores": 16,
    "rows": 17,
}


def _rng(seed: int, name: str, layer: int = 0, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), _TENSOR_IDS[name], int(layer), int(extra)])


def _normal(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return round_bf16(a) if dtype == "bf16" else a


def layer_weights(dims: ModelDims, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """Weights of one transformer block, N(0, 0.02); norm gains are 1, no biases.

    Layouts are [out_features, in_features]: wqkv rows are Q (d_q), then K (d_kv),
    then V (d_kv); w_gate_up rows are the gate (d_ffn) then the up projection."""
    d, dq, dkv, f = dims.d_model, dims.d_q, dims.d_kv, dims.d_ffn
    return {
        "attn_norm": np.ones(d, np.float32),
        "wqkv": _normal(_rng(seed, "wqkv", layer), (dq + 2 * dkv, d), 0.02, dims.dtype),
        "wo": _normal(_rng(seed, "wo", layer), (d, dq), 0.02, dims.dtype),
        "ffn_norm": np.ones(d, np.float32),
        "w_gate_up": _normal(_rng(seed, "w_gate_up", layer), (2 * f, d), 0.02, dims.dtype),
        "w_down": _normal(_rng(seed, "w_down", layer), (d, f), 0.02, dims.dtype),
    }


def embedding_rows(dims: ModelDims, seed: int, vocab: Optional[int] = None) -> np.ndarray:
    v = dims.vocab if vocab is None else vocab
    return _normal(_rng(seed, "tok_emb"), (v, dims.d_model), 0.02, dims.dtype)


def lm_head(dims: ModelDims, seed: int) -> np.ndarray:
    return _normal(_rng(seed, "lm_head"), (dims.vocab, dims.d_model), 0.02, dims.dtype)


def model_weights(dims: ModelDims, seed: int, layers: Optional[Iterable[int]] = None) -> Dict:
    """Full weight set {tok_emb, final_norm, lm_head, layers: [..]}.

    `layers` selects which block indices to draw (default: all n_layers); the
    returned model then has len(layers) blocks, in the given order."""
    ls = list(range(dims.n_layers)) if layers is None else list(layers)
    return {
        "tok_emb": embedding_rows(dims, seed),
        "final_norm": np.ones(dims.d_model, np.float32),
        "lm_head": lm_head(dims, seed),
        "layers": [layer_weights(dims, seed, l) for l in ls],
    }


def with_layers(dims: ModelDims, n_layers: int) -> ModelDims:
    return replace(dims, n_layers=n_layers)


def prompt_tokens(dims: ModelDims, prompt_len: int, seed: int, seq: int = 0) -> np.ndarray:
    """Uniform random prompt ids on [0, vocab) excluding the [MASK] id."""
    return _rng(seed, "prompt", 0, seq).integers(0, dims.vocab - 1, size=prompt_len).astype(np.int32)


def initial_sequence(dims: ModelDims, setup: DecodeSetup, seed: int, seq: int = 0):
    """y_0 = prompt followed by gen_len [MASK] ids, and the mask flags (Sec. 3.1)."""
    y = np.full(setup.seq_len, dims.mask_id, np.int32)
    y[: setup.prompt_len] = prompt_tokens(dims, setup.prompt_len, seed, seq)
    is_masked = np.zeros(setup.seq_len, np.uint8)
    is_masked[setup.prompt_len:] = 1
    return y, is_masked


def distinct_sorted_rows(seed: int, L: int, m: int, extra: int = 0) -> np.ndarray:
    """m distinct positions of 0..L-1, ascending: the first m entries of a seeded permutation."""
    perm = _rng(seed, "attn_idx", 0, extra).permutation(L)
    return np.sort(perm[:m]).astype(np.int32)


def attention_case(seed: int, n_heads: int, n_kv_heads: int, head_dim: int, L: int, m: int,
                   dtype: str = "bf16") -> Dict[str, np.ndarray]:
    """Isolated selective-refresh attention op: cached K/V ~ N(0,1) of length L,
    m query rows and m new K/V rows at seeded distinct positions."""
    dkv = n_kv_heads * head_dim
    return {
        "q": _normal(_rng(seed, "attn_q"), (m, n_heads * head_dim), 1.0, dtype),
        "k_cache": _normal(_rng(seed, "attn_k"), (L, dkv), 1.0, dtype),
        "v_cache": _normal(_rng(seed, "attn_v"), (L, dkv), 1.0, dtype),
        "new_k": _normal(_rng(seed, "attn_newk"), (m, dkv), 1.0, dtype),
        "new_v": _normal(_rng(seed, "attn_newv"), (m, dkv), 1.0, dtype),
        "idx": distinct_sorted_rows(seed, L, m),
    }


def hidden_rows(seed: int, m: int, d: int, std: float = 1.0, extra: int = 0) -> np.ndarray:
    return _rng(seed, "hidden", 0, extra).standard_normal(size=(m, d), dtype=np.float32) * np.float32(std)


def logits_rows(seed: int, rows: int, vocab: int, std: float = 2.0, extra: int = 0) -> np.ndarray:
    return _rng(seed, "logits", 0, extra).standard_normal(size=(rows, vocab), dtype=np.float32) * np.float32(std)


def skewed_influence(seed: int, L: int, n_sinks: int = 4, extra: int = 0) -> np.ndarray:
    """Influence scores shaped like a trained dLLM's rollout column sums: a few
    sink positions carry most of the mass, the rest a Zipf-like tail; sums to L."""
    rng = _rng(seed, "scores", 0, extra)
    c = 1.0 / (1.0 + rng.permutation(L).astype(np.float64))
    sinks = rng.choice(L, size=min(n_sinks, L), replace=False)
    c[sinks] += 0.5 * L / max(1, len(sinks))
    c *= L / c.sum()
    return c.astype(np.float32)


def random_scores(seed: int, n: int, extra: int = 0) -> np.ndarray:
    return _rng(seed, "scores", 1, extra).random(size=n, dtype=np.float32)


def random_mask(seed: int, L: int, prompt_len: int, frac_known: float, extra: int = 0) -> np.ndarray:
    """Mask flags of a partly decoded sequence: prompt known, each generation
    slot known with probability frac_known."""
    rng = _rng(seed, "rows", 0, extra)
    is_masked = np.zeros(L, np.uint8)
    is_masked[prompt_len:] = (rng.random(L - prompt_len) >= frac_known).astype(np.uint8)
    return is_masked
