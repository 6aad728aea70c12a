"""ctypes binding of libd2c.so: the same names as the C ABI (include/d2c.h),
argument marshalling only.  PyTorch supplies device memory and the stream; every
step of the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing, importing this module raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libd2c.so")

D2C_OK, D2C_EINVAL, D2C_ENOMEM, D2C_EHIP, D2C_ESHAPE = 0, -1, -2, -3, -4
D2C_F32, D2C_BF16 = 0, 1
D2C_STATIC_MAX_ROWS = 256
CNT_MSTAR, CNT_U, CNT_S, CNT_DECODE, CNT_NEXT_ROWS, CNT_MASKED, CNT_BLOCK_LO, CNT_BLOCK_HI, N_COUNTS = range(9)


PROF_CLASSES = ("gemm", "attention", "rollout", "rowwise", "select", "attn_avg")


class D2CError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("d2c error %d: %s" % (code, msg))
        self.code = code


class d2c_dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn",
                                          "vocab", "max_seq", "dtype")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("mask_id", C.c_int32), ("max_batch", C.c_int32)]


class d2c_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("bqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("ffn_norm", C.POINTER(C.c_void_p)), ("w_gate_up", C.POINTER(C.c_void_p)),
                ("w_down", C.POINTER(C.c_void_p))]


class d2c_params(C.Structure):
    _fields_ = [("sigma", C.c_float), ("k", C.c_int32), ("p", C.c_float), ("block_len", C.c_int32),
                ("n_unmask", C.c_int32), ("cand_mode", C.c_int32), ("threshold", C.c_float),
                ("conf_decode", C.c_int32), ("rollout_layers", C.c_int32)]


class d2c_seq_state(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("tokens", "is_masked", "k_cache", "v_cache", "conf", "pred", "s_idx",
                                          "s_rows", "influence", "mstar", "u_set", "decode_idx", "counts",
                                          "score", "hidden_out", "logits_out")] + \
               [(n, C.c_int32) for n in ("L", "prompt_len", "n_s", "n_rows", "n_masked", "step")]


class d2c_tunable(C.Structure):
    _fields_ = [("name", C.c_char_p), ("value", C.c_int32)]


# include/d2c.h (the method's calls) and include/d2c_tools.h (timing, tunables, planner)
EXPORTS = ["d2c_init", "d2c_destroy", "d2c_last_error", "d2c_seq_reset", "d2c_select", "d2c_refresh_layer",
           "d2c_attention", "d2c_influence", "d2c_linear", "d2c_step", "d2c_workspace_bytes", "d2c_select_static"]
TOOL_EXPORTS = ["d2c_profile_begin", "d2c_profile_end", "d2c_init_tuned", "d2c_ctx_set_tunable",
                "d2c_plan_projection", "d2c_memory_info"]


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libd2c.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_2509_23094_amd/build.py) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.d2c_init.argtypes = [C.POINTER(d2c_dims), C.POINTER(d2c_weights), C.POINTER(vp)]
    lib.d2c_destroy.argtypes = [vp]
    lib.d2c_last_error.argtypes = [vp]
    lib.d2c_last_error.restype = C.c_char_p
    lib.d2c_seq_reset.argtypes = [vp, C.POINTER(d2c_seq_state), vp]
    lib.d2c_select.argtypes = [vp, C.POINTER(d2c_params), vp, vp, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp,
                               vp, vp, vp, vp]
    lib.d2c_select_static.argtypes = [C.POINTER(d2c_params), i32, vp, vp, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp,
                                      vp, vp, vp, vp, vp, vp]
    lib.d2c_refresh_layer.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
    lib.d2c_attention.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.d2c_influence.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.d2c_linear.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    lib.d2c_step.argtypes = [vp, C.POINTER(d2c_params), C.POINTER(d2c_seq_state), i32, vp]
    lib.d2c_profile_begin.argtypes = [vp]
    lib.d2c_profile_end.argtypes = [vp, vp, vp, vp]
    lib.d2c_workspace_bytes.argtypes = [vp]
    lib.d2c_workspace_bytes.restype = C.c_int64
    lib.d2c_init_tuned.argtypes = [C.POINTER(d2c_dims), C.POINTER(d2c_weights), C.POINTER(d2c_tunable), i32,
                                   C.POINTER(vp)]
    lib.d2c_ctx_set_tunable.argtypes = [vp, C.c_char_p, i32]
    lib.d2c_memory_info.argtypes = [vp, C.POINTER(C.c_int64)]
    lib.d2c_plan_projection.argtypes = [i32, i32, i32, i32, i32, C.POINTER(i32)]
    for name in EXPORTS + TOOL_EXPORTS:
        if name not in ("d2c_last_error", "d2c_workspace_bytes"):
            getattr(lib, name).restype = C.c_int
    return lib


_lib = load_library()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def torch_dtype(dtype: str) -> torch.dtype:
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    """numpy float32 -> device tensor of the storage type (exact for bf16-representable values)."""
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch_dtype(dtype)).cuda().contiguous()


def d2c_plan_projection(dtype: str, m: int, N: int, K: int, single_split: bool = False) -> Dict[str, int]:
    """Launch shape of the projection kernel for m rows of a [N, K] matrix (host arithmetic, no GPU)."""
    shape = (C.c_int32 * 7)()
    rc = _lib.d2c_plan_projection(D2C_BF16 if dtype == "bf16" else D2C_F32, int(m), int(N), int(K), int(single_split), shape)
    if rc != 0:
        raise D2CError(rc, "d2c_plan_projection: bad arguments")
    return dict(zip(("row_tiles", "col_tiles_per_wave", "waves", "splits", "k_per_split", "row_chunks", "workgroups"),
                    [int(x) for x in shape]))


def make_params(sigma=10.0, k=32, p=0.1, block_len=32, n_unmask=1, cand_mode=0, threshold=0.0, conf_decode=0,
                rollout_layers=0) -> d2c_params:
    return d2c_params(float(sigma), int(k), float(p), int(block_len), int(n_unmask), int(cand_mode),
                      float(threshold), int(conf_decode), int(rollout_layers))


def d2c_select_static(params: d2c_params, vocab: int, logits, logit_pos, n_rows, tokens, is_masked, L, prompt_len,
                      conf, pred, influence, mstar, u_set, decode_idx, s_next, s_rows_next, counts,
                      score_out=None) -> None:
    """d2c_select without a context and without any allocation (scratch in a static device array)."""
    rc = _lib.d2c_select_static(C.byref(params), int(vocab), _ptr(logits), _ptr(logit_pos), n_rows, _ptr(tokens),
                                _ptr(is_masked), L, prompt_len, _ptr(conf), _ptr(pred), _ptr(influence), _ptr(mstar),
                                _ptr(u_set), _ptr(decode_idx), _ptr(s_next), _ptr(s_rows_next), _ptr(counts),
                                _ptr(score_out), _stream())
    if rc != D2C_OK:
        raise D2CError(rc, (_lib.d2c_last_error(None) or b"").decode())


class Context:
    """Owns a d2c_ctx and keeps the borrowed weight tensors alive."""

    def __init__(self, dims, weights: Dict, max_seq: int, device_weights: bool = False, max_batch: int = 1,
                 tunables: Optional[Dict[str, int]] = None):
        """dims: workloads.ModelDims; weights: {tok_emb, final_norm, lm_head, layers: [{...}]} as numpy
        float32 arrays, or (device_weights=True) as device tensors already in the storage type.
        tunables: launch-shape tunables of this context (d2c_tools.h), in force from d2c_init_tuned on."""
        self.dims = dims
        self.dtype = dims.dtype
        self.max_seq = int(max_seq)
        n_layers = len(weights["layers"])
        self._keep: List[torch.Tensor] = []

        def dev(a, storage):
            if device_weights:
                t = a
            elif storage:
                t = to_device(a, self.dtype)
            else:
                t = torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()
            assert t.is_cuda and t.is_contiguous()
            assert t.dtype == (torch_dtype(self.dtype) if storage else torch.float32)
            self._keep.append(t)
            return t

        self.tok_emb = dev(weights["tok_emb"], True)
        self.final_norm = dev(weights["final_norm"], False)
        self.lm_head = dev(weights["lm_head"], True)
        per_layer = {k: [] for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}
        has_bias = weights["layers"][0].get("bqkv") is not None
        bias = []
        for lw in weights["layers"]:
            for k in per_layer:
                per_layer[k].append(dev(lw[k], k not in ("attn_norm", "ffn_norm")))
            if has_bias:
                bias.append(dev(lw["bqkv"], False))
        self.layers = per_layer

        def arr(ts):
            a = (C.c_void_p * n_layers)(*[t.data_ptr() for t in ts])
            self._keep.append(a)
            return a

        w = d2c_weights()
        w.tok_emb, w.final_norm, w.lm_head = self.tok_emb.data_ptr(), self.final_norm.data_ptr(), self.lm_head.data_ptr()
        for k in per_layer:
            setattr(w, k, arr(per_layer[k]))
        w.bqkv = arr(bias) if has_bias else None
        d = d2c_dims(n_layers, dims.d_model, dims.n_heads, dims.n_kv_heads, dims.head_dim, dims.d_ffn, dims.vocab,
                     self.max_seq, D2C_BF16 if self.dtype == "bf16" else D2C_F32, dims.rms_eps, dims.rope_theta,
                     dims.mask_id, int(max_batch))
        self.n_layers = n_layers
        self.handle = C.c_void_p()
        tun = sorted((tunables or {}).items())
        names = [k.encode() for k, _ in tun]
        arr_t = (d2c_tunable * max(1, len(tun)))(*[d2c_tunable(n, int(v)) for n, (_, v) in zip(names, tun)])
        rc = _lib.d2c_init_tuned(C.byref(d), C.byref(w), arr_t, len(tun), C.byref(self.handle))
        if rc != D2C_OK:
            raise D2CError(rc, (_lib.d2c_last_error(None) or b"").decode())

    def _check(self, rc: int) -> None:
        if rc != D2C_OK:
            raise D2CError(rc, (_lib.d2c_last_error(self.handle) or b"").decode())

    def close(self) -> None:
        if self.handle:
            _lib.d2c_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self) -> int:
        return int(_lib.d2c_workspace_bytes(self.handle))

    def set_tunable(self, name: str, value: int) -> None:
        self._check(_lib.d2c_ctx_set_tunable(self.handle, name.encode(), int(value)))

    def memory_info(self) -> Dict[str, int]:
        b = (C.c_int64 * 4)()
        self._check(_lib.d2c_memory_info(self.handle, b))
        return dict(zip(("total_bytes", "pretiled_weight_bytes", "rollout_bytes", "attention_scratch_bytes"),
                        [int(x) for x in b]))

    # ------------------------------------------------------------------ C ABI calls
    def d2c_refresh_layer(self, layer: int, hidden: torch.Tensor, idx: torch.Tensor, idx_host: np.ndarray,
                          k_cache: torch.Tensor, v_cache: torch.Tensor, L: int,
                          attn_avg: Optional[torch.Tensor] = None, rollout: Optional[torch.Tensor] = None,
                          m: Optional[int] = None) -> None:
        idx_host = np.ascontiguousarray(idx_host, np.int32)
        m = len(idx_host) if m is None else m
        self._check(_lib.d2c_refresh_layer(self.handle, layer, _ptr(hidden), _ptr(idx),
                                           idx_host.ctypes.data_as(C.c_void_p), m, _ptr(k_cache), _ptr(v_cache), L,
                                           _ptr(attn_avg), _ptr(rollout), _stream()))

    def d2c_attention(self, q, idx, m, new_k, new_v, k_cache, v_cache, L, out, attn_avg=None) -> None:
        self._check(_lib.d2c_attention(self.handle, _ptr(q), _ptr(idx), m, _ptr(new_k), _ptr(new_v), _ptr(k_cache),
                                       _ptr(v_cache), L, _ptr(out), _ptr(attn_avg), _stream()))

    def d2c_profile_begin(self) -> None:
        self._check(_lib.d2c_profile_begin(self.handle))

    def d2c_profile_end(self) -> Dict[str, Dict[str, float]]:
        n = len(PROF_CLASSES)
        ms, cnt, by = (C.c_double * n)(), (C.c_int64 * n)(), (C.c_double * n)()
        self._check(_lib.d2c_profile_end(self.handle, ms, cnt, by))
        return {name: {"ms": ms[i], "launches": int(cnt[i]), "bytes": by[i]} for i, name in enumerate(PROF_CLASSES)}

    def d2c_linear(self, a, w, m, N, K, out) -> None:
        self._check(_lib.d2c_linear(self.handle, _ptr(a), _ptr(w), m, N, K, _ptr(out), _stream()))

    def d2c_influence(self, rollout, idx, m, L, influence) -> None:
        self._check(_lib.d2c_influence(self.handle, _ptr(rollout), _ptr(idx), m, L, _ptr(influence), _stream()))

    def d2c_select(self, params: d2c_params, logits, logit_pos, n_rows, tokens, is_masked, L, prompt_len, conf, pred,
                   influence, mstar, u_set, decode_idx, s_next, s_rows_next, counts, score_out=None) -> None:
        self._check(_lib.d2c_select(self.handle, C.byref(params), _ptr(logits), _ptr(logit_pos), n_rows, _ptr(tokens),
                                    _ptr(is_masked), L, prompt_len, _ptr(conf), _ptr(pred), _ptr(influence),
                                    _ptr(mstar), _ptr(u_set), _ptr(decode_idx), _ptr(s_next), _ptr(s_rows_next),
                                    _ptr(counts), _ptr(score_out), _stream()))

    def d2c_seq_reset(self, seq: "Sequence_") -> None:
        self._check(_lib.d2c_seq_reset(self.handle, C.byref(seq.c), _stream()))

    def d2c_step(self, params: d2c_params, seqs: Sequence["Sequence_"]) -> None:
        arr = (d2c_seq_state * len(seqs))(*[s.c for s in seqs])
        rc = _lib.d2c_step(self.handle, C.byref(params), arr, len(seqs), _stream())
        for s, c in zip(seqs, arr):
            s.c.n_s, s.c.n_rows, s.c.n_masked, s.c.step = c.n_s, c.n_rows, c.n_masked, c.step
        self._check(rc)


class Sequence_:
    """Device buffers of one sequence's decoding state (allocated with torch) and the C struct over them."""

    def __init__(self, ctx: Context, tokens: np.ndarray, is_masked: np.ndarray, prompt_len: int,
                 trace: bool = False, max_trace_rows: Optional[int] = None):
        L = len(tokens)
        dims = ctx.dims
        dev = "cuda"
        self.L, self.prompt_len = L, int(prompt_len)
        self.tokens = torch.from_numpy(np.ascontiguousarray(tokens, np.int32)).to(dev)
        self.is_masked = torch.from_numpy(np.ascontiguousarray(is_masked, np.uint8)).to(dev)
        tdt = torch_dtype(ctx.dtype)
        self.k_cache = torch.zeros((ctx.n_layers, L, dims.d_kv), dtype=tdt, device=dev)
        self.v_cache = torch.zeros((ctx.n_layers, L, dims.d_kv), dtype=tdt, device=dev)
        self.conf = torch.zeros(L, dtype=torch.float32, device=dev)
        self.pred = torch.zeros(L, dtype=torch.int32, device=dev)
        self.s_idx = torch.zeros(L, dtype=torch.int32, device=dev)
        self.s_rows = torch.zeros(L, dtype=torch.int32, device=dev)
        self.influence = torch.zeros(L, dtype=torch.float32, device=dev)
        self.mstar = torch.zeros(L, dtype=torch.int32, device=dev)
        self.u_set = torch.zeros(L, dtype=torch.int32, device=dev)
        self.decode_idx = torch.zeros(L, dtype=torch.int32, device=dev)
        self.counts = torch.zeros(N_COUNTS, dtype=torch.int32, device=dev)
        self.score = torch.zeros(L, dtype=torch.float32, device=dev) if trace else None
        self.hidden_out = torch.zeros((L, dims.d_model), dtype=torch.float32, device=dev) if trace else None
        rows = L if max_trace_rows is None else max_trace_rows
        self.logits_out = torch.zeros((rows, dims.vocab), dtype=torch.float32, device=dev) if trace else None
        c = d2c_seq_state()
        for name in ("tokens", "is_masked", "k_cache", "v_cache", "conf", "pred", "s_idx", "s_rows", "influence",
                     "mstar", "u_set", "decode_idx", "counts", "score", "hidden_out", "logits_out"):
            setattr(c, name, _ptr(getattr(self, name)))
        c.L, c.prompt_len = L, self.prompt_len
        self.c = c
        ctx.d2c_seq_reset(self)

    @property
    def n_s(self) -> int:
        return self.c.n_s

    @property
    def n_rows(self) -> int:
        return self.c.n_rows

    @property
    def n_masked(self) -> int:
        return self.c.n_masked

    def set_selection(self, s_idx: np.ndarray, s_rows: np.ndarray) -> None:
        """Overwrite S_t (teacher forcing): s_idx ascending positions, s_rows its still-masked compact rows."""
        self.s_idx[: len(s_idx)] = torch.from_numpy(np.ascontiguousarray(s_idx, np.int32)).cuda()
        self.s_rows[: len(s_rows)] = torch.from_numpy(np.ascontiguousarray(s_rows, np.int32)).cuda()
        self.c.n_s, self.c.n_rows = len(s_idx), len(s_rows)
