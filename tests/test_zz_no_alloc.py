"""d2c_select_static -- the selection call that allocates nothing (its scratch is a static device array inside
the library) -- against d2c_select on the same inputs: two calls in a row, the second on a smaller input, so
that whatever the first call left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2509_23094_amd import workloads as W

from gpu_util import say

pytestmark = pytest.mark.gpu

OUT_NAMES = ("mstar", "u_set", "decode_idx", "s_next", "s_rows_next")


def _inputs(L, P, V, n_rows, seed):
    is_masked = W.random_mask(seed, L, P, 0.4).astype(bool)
    y = np.where(is_masked, V - 1, 7).astype(np.int32)
    conf = W.random_scores(seed, L)
    pred = (np.arange(L) * 5 % V).astype(np.int32)
    c = W.skewed_influence(seed, L)
    pos = np.flatnonzero(is_masked)[:: 2][:n_rows].astype(np.int32)
    logits = W.logits_rows(seed, len(pos), V)
    if len(pos) > 1:
        logits[1, 9] = logits[1, 4] = logits[1].max() + 1.0          # tied maxima: the lowest index wins
    return y, is_masked, conf, pred, c, pos, logits


def _device_state(B, L, y, is_masked, conf, pred, c):
    t = {"tokens": torch.from_numpy(y.copy()).cuda(), "is_masked": torch.from_numpy(is_masked.astype(np.uint8)).cuda(),
         "conf": torch.from_numpy(conf.copy()).cuda(), "pred": torch.from_numpy(pred.copy()).cuda(),
         "influence": torch.from_numpy(c.copy()).cuda(),
         "counts": torch.full((B.N_COUNTS,), -7, dtype=torch.int32, device="cuda"),
         "score": torch.full((L,), -7.0, dtype=torch.float32, device="cuda")}
    for name in OUT_NAMES:
        t[name] = torch.full((L,), -1, dtype=torch.int32, device="cuda")
    return t


def test_select_static_matches_select_on_two_calls_in_a_row():
    from paper_2509_23094_amd import binding as B
    V = 126464                                                         # LLaDA's vocabulary: 16 chunks per row
    cases = [(512, 256, 40, 3), (96, 32, 5, 4)]                        # (L, prompt, logit rows, seed): large, then small
    wd = W.ModelDims(1, 64, 4, 4, 16, 80, V, dtype="f32")
    mdl = W.model_weights(W.ModelDims(1, 64, 4, 4, 16, 80, 8, dtype="f32"), 0)
    mdl["tok_emb"] = mdl["lm_head"] = np.zeros((V, 64), np.float32)     # the selection never reads them
    ctx = B.Context(wd, mdl, 512)
    prm = B.make_params(10.0, 32, 0.1, 32, 2, 0, 0.9, 0)
    # reference results first (d2c_select with a context), then the two static calls back to back
    refs, devs = [], []
    for L, P, n_rows, seed in cases:
        y, is_masked, conf, pred, c, pos, logits = _inputs(L, P, V, n_rows, seed)
        lg, lp = torch.from_numpy(logits).cuda(), torch.from_numpy(pos).cuda()
        r = _device_state(B, L, y, is_masked, conf, pred, c)
        say(f"d2c_select (reference) L={L} rows={len(pos)}")
        ctx.d2c_select(prm, lg, lp, len(pos), r["tokens"], r["is_masked"], L, P, r["conf"], r["pred"], r["influence"],
                       r["mstar"], r["u_set"], r["decode_idx"], r["s_next"], r["s_rows_next"], r["counts"], r["score"])
        refs.append(r)
        devs.append((L, P, lg, lp, len(pos), _device_state(B, L, y, is_masked, conf, pred, c)))
    torch.cuda.synchronize()
    for L, P, lg, lp, n, t in devs:                                     # no synchronisation between the two calls
        say(f"d2c_select_static L={L} rows={n}")
        B.d2c_select_static(prm, V, lg, lp, n, t["tokens"], t["is_masked"], L, P, t["conf"], t["pred"], t["influence"],
                            t["mstar"], t["u_set"], t["decode_idx"], t["s_next"], t["s_rows_next"], t["counts"],
                            t["score"])
    torch.cuda.synchronize()
    for (L, P, lg, lp, n, t), r in zip(devs, refs):
        assert int(r["counts"][B.CNT_S]) > 0 and int(r["counts"][B.CNT_DECODE]) >= 2
        for name in ("tokens", "is_masked", "conf", "pred", "counts", "score") + OUT_NAMES:
            assert torch.equal(t[name], r[name]), f"{name} differs at L={L}"       # same kernels: same bits
    # limits are refused with a clear error and nothing is launched
    L, P, lg, lp, n, t = devs[0]
    with pytest.raises(B.D2CError) as ei:
        B.d2c_select_static(prm, V, lg, lp, B.D2C_STATIC_MAX_ROWS + 1, t["tokens"], t["is_masked"], L, P, t["conf"],
                            t["pred"], t["influence"], t["mstar"], t["u_set"], t["decode_idx"], t["s_next"],
                            t["s_rows_next"], t["counts"], t["score"])
    assert ei.value.code == B.D2C_ESHAPE and "D2C_STATIC_MAX_ROWS" in str(ei.value)
    with pytest.raises(B.D2CError) as ei:
        B.d2c_select_static(prm, V, lg, lp, n, t["tokens"], t["is_masked"], 4097, P, t["conf"], t["pred"],
                            t["influence"], t["mstar"], t["u_set"], t["decode_idx"], t["s_next"], t["s_rows_next"],
                            t["counts"], t["score"])
    assert ei.value.code == B.D2C_ESHAPE
    ctx.close()
