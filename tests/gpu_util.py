"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import sys

import numpy as np

from oracle import d2cache_oracle as O
from paper_2509_23094_amd import workloads as W

# Tolerances of the parity bar: relative L2 error against the fp64 oracle.
TOL = {"f32": 1e-5, "bf16": 2e-2}


def say(msg: str) -> None:
    """Name the case before each GPU step, flushed, so that a fault can be attributed."""
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def oracle_dims(wd: W.ModelDims, n_layers=None) -> O.Dims:
    return O.Dims(wd.n_layers if n_layers is None else n_layers, wd.d_model, wd.n_heads, wd.n_kv_heads,
                  wd.head_dim, wd.d_ffn, wd.vocab, wd.rms_eps, wd.rope_theta)


def oracle_params(su: W.DecodeSetup, **over) -> O.Params:
    kw = dict(sigma=su.sigma, k=su.k, p=su.p, block_len=su.block_len, n_unmask=su.n_unmask)
    kw.update(over)
    return O.Params(**kw)


def rel_l2(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.sqrt((ref * ref).sum())
    return float(np.sqrt(((got - ref) ** 2).sum()) / (den if den > 0 else 1.0))


def host(t) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def topk_margin(score: np.ndarray, cand: np.ndarray, k: int) -> float:
    """Relative gap between the k-th and (k+1)-th largest candidate scores (inf if all are taken)."""
    if k <= 0 or len(cand) <= k:
        return float("inf")
    s = np.sort(np.asarray(score, np.float64)[cand])[::-1]
    return float((s[k - 1] - s[k]) / max(abs(s[k - 1]), 1e-300))


def topp_margin(c: np.ndarray, cand: np.ndarray, p: float) -> float:
    """How far the stage-2 cut is from flipping, relative to the candidates' total mass: the distance
    of the cumulative mass from p on both sides of the cut, and the gap between the last member taken
    and the first one left out."""
    if len(cand) == 0 or p >= 1.0:
        return float("inf")
    v = np.sort(np.asarray(c, np.float64)[cand])[::-1]
    tot = v.sum()
    cum = np.cumsum(v) / tot
    over = np.flatnonzero(cum > p)
    if len(over) == 0:
        return float("inf")
    take = int(over[0]) + 1
    gaps = [cum[take - 1] - p]
    if take >= 2:
        gaps.append(p - cum[take - 2])
    if take < len(v):
        gaps.append((v[take - 1] - v[take]) / tot)
    return float(min(gaps))
