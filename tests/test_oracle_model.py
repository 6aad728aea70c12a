"""Pins for the oracle's partial forward and step loop (Sec. 3.1, Eq. 5, Sec. 4.2).

Library witnesses (torch CPU, fp64), invariants, and the three whole-step
checks: select-all == full recomputation, select-none leaves the cache alone,
and a scalar brute force on a tiny model."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import d2cache_oracle as O
from paper_2509_23094_amd import workloads as W

from brute_force import brute_influence, brute_step


def _dims(wd: W.ModelDims) -> O.Dims:
    return O.Dims(wd.n_layers, wd.d_model, wd.n_heads, wd.n_kv_heads, wd.head_dim, wd.d_ffn,
                  wd.vocab, wd.rms_eps, wd.rope_theta)


TINY = W.ModelDims(2, 32, 4, 2, 8, 48, 40, dtype="f32")      # GQA 4/2
TINY_SETUP = W.DecodeSetup(6, 10, 5, 1, k=3, p=0.5, sigma=2.0)


def _tiny_model(seed=0, wd=TINY, std_scale=8.0):
    mdl = W.model_weights(wd, seed)
    # N(0, 0.02) weights give nearly uniform attention; widen them so that the
    # pins see structured attention and decisive logits.
    for k in ("tok_emb", "lm_head"):
        mdl[k] = mdl[k] * np.float32(std_scale)
    for lw in mdl["layers"]:
        for k in ("wqkv", "wo", "w_gate_up", "w_down"):
            lw[k] = lw[k] * np.float32(std_scale)
        lw["attn_norm"] = 1.0 + 0.1 * W.hidden_rows(seed, 1, wd.d_model, extra=1)[0]
        lw["ffn_norm"] = 1.0 + 0.1 * W.hidden_rows(seed, 1, wd.d_model, extra=2)[0]
    mdl["final_norm"] = 1.0 + 0.1 * W.hidden_rows(seed, 1, wd.d_model, extra=3)[0]
    return mdl


# ---------------------------------------------------------------- pieces
def test_rmsnorm_library_witness_and_unit_rms():
    x = W.hidden_rows(0, 5, 64).astype(np.float64)
    g = 1.0 + 0.2 * W.hidden_rows(1, 1, 64)[0].astype(np.float64)
    got = O.rmsnorm(x, g, 1e-5)
    ref = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-13)
    unit = O.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((unit ** 2).mean(axis=1)), 1.0, rtol=1e-14)
    np.testing.assert_allclose(O.rmsnorm(3.0 * x, g, 0.0), O.rmsnorm(x, g, 0.0), rtol=1e-13)


def test_rope_properties():
    dh, theta = 16, 10000.0
    q = W.hidden_rows(2, 6, 2 * dh).astype(np.float64).reshape(6, 2, dh)
    k = W.hidden_rows(3, 6, 2 * dh).astype(np.float64).reshape(6, 2, dh)
    pos = np.array([0, 1, 5, 17, 100, 511])
    rq = O.rope(q, pos, theta)
    np.testing.assert_array_equal(rq[0], q[0])                       # position 0: identity
    np.testing.assert_allclose((rq ** 2).sum(-1), (q ** 2).sum(-1), rtol=1e-13)   # a rotation
    # relative-position property: <R_i q, R_j k> depends on i - j only
    a = O.rope(q[:1], np.array([7]), theta)[0, 0] @ O.rope(k[:1], np.array([3]), theta)[0, 0]
    b = O.rope(q[:1], np.array([104]), theta)[0, 0] @ O.rope(k[:1], np.array([100]), theta)[0, 0]
    assert abs(a - b) < 1e-11
    # complex-number witness: pair (x_i, x_{i+dh/2}) is multiplied by exp(i pos theta^{-2i/dh})
    half = dh // 2
    for r, p in enumerate(pos):
        z = (q[r, 1, :half] + 1j * q[r, 1, half:]) * np.exp(1j * p * theta ** (-2.0 * np.arange(half) / dh))
        np.testing.assert_allclose(rq[r, 1, :half], z.real, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(rq[r, 1, half:], z.imag, rtol=1e-12, atol=1e-13)


def test_attention_library_witness_full_rows():
    # m = L, every row a query: plain softmax(Q K^T / sqrt(d_h)) V, with GQA
    H, Hkv, dh, L = 4, 2, 8, 19
    case = W.attention_case(0, H, Hkv, dh, L, L, dtype="f32")
    out, abar = O.selective_attention(case["q"], case["k_cache"], case["v_cache"], H, Hkv, dh)
    q = torch.from_numpy(case["q"].astype(np.float64)).view(L, H, dh).transpose(0, 1)
    k = torch.from_numpy(case["k_cache"].astype(np.float64)).view(L, Hkv, dh).transpose(0, 1)
    v = torch.from_numpy(case["v_cache"].astype(np.float64)).view(L, Hkv, dh).transpose(0, 1)
    k, v = k.repeat_interleave(H // Hkv, 0), v.repeat_interleave(H // Hkv, 0)
    ref = F.scaled_dot_product_attention(q, k, v).transpose(0, 1).reshape(L, H * dh).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(abar.sum(axis=1), 1.0, atol=1e-14)
    probs = torch.softmax(q @ k.transpose(1, 2) / math.sqrt(dh), dim=-1).mean(0).numpy()
    np.testing.assert_allclose(abar, probs, rtol=1e-11, atol=1e-14)


def test_attention_key_permutation_permutes_abar_columns():
    H, Hkv, dh, L, m = 2, 2, 8, 12, 5
    case = W.attention_case(1, H, Hkv, dh, L, m, dtype="f32")
    out, abar = O.selective_attention(case["q"], case["k_cache"], case["v_cache"], H, Hkv, dh)
    perm = np.random.default_rng(0).permutation(L)
    out2, abar2 = O.selective_attention(case["q"], case["k_cache"][perm], case["v_cache"][perm], H, Hkv, dh)
    np.testing.assert_allclose(out2, out, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(abar2, abar[:, perm], rtol=1e-12, atol=1e-15)


def test_refresh_layer_library_witness():
    # one block, rows S of a longer cache, re-done with torch's own routines
    wd, L, m = TINY, 14, 6
    dims = _dims(wd)
    mdl = _tiny_model(3)
    w = mdl["layers"][0]
    S = W.distinct_sorted_rows(4, L, m)
    h = W.hidden_rows(5, m, wd.d_model)
    kc = W.hidden_rows(6, L, wd.d_kv).astype(np.float64)
    vc = W.hidden_rows(7, L, wd.d_kv).astype(np.float64)
    kc0, vc0 = kc.copy(), vc.copy()
    h_new, abar = O.refresh_layer(dims, w, h, S, kc, vc)

    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    H, Hkv, dh = wd.n_heads, wd.n_kv_heads, wd.head_dim
    x = t(h)
    a = F.rms_norm(x, (wd.d_model,), t(w["attn_norm"]), eps=wd.rms_eps)
    qkv = F.linear(a, t(w["wqkv"]))
    q, k, v = qkv.split([H * dh, Hkv * dh, Hkv * dh], dim=-1)

    def rot(z, nh):
        z = z.view(m, nh, dh)
        zc = torch.complex(z[..., : dh // 2], z[..., dh // 2:])
        ang = t(S)[:, None] * wd.rope_theta ** (-2.0 * torch.arange(dh // 2, dtype=torch.float64) / dh)
        zc = zc * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([zc.real, zc.imag], dim=-1)

    q, k = rot(q, H), rot(k, Hkv)
    K, V = t(kc0).view(L, Hkv, dh).clone(), t(vc0).view(L, Hkv, dh).clone()
    K[torch.from_numpy(S).long()] = k
    V[torch.from_numpy(S).long()] = v.view(m, Hkv, dh)
    att = F.scaled_dot_product_attention(q.transpose(0, 1), K.transpose(0, 1).repeat_interleave(H // Hkv, 0),
                                         V.transpose(0, 1).repeat_interleave(H // Hkv, 0))
    x = x + F.linear(att.transpose(0, 1).reshape(m, H * dh), t(w["wo"]))
    b = F.rms_norm(x, (wd.d_model,), t(w["ffn_norm"]), eps=wd.rms_eps)
    g, u = F.linear(b, t(w["w_gate_up"])).split([wd.d_ffn, wd.d_ffn], dim=-1)
    x = x + F.linear(F.silu(g) * u, t(w["w_down"]))
    np.testing.assert_allclose(h_new, x.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(kc, K.view(L, -1).numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(vc, V.view(L, -1).numpy(), rtol=1e-12, atol=1e-13)
    untouched = np.setdiff1d(np.arange(L), S)
    np.testing.assert_array_equal(kc[untouched], kc0[untouched])       # reused rows are not rewritten
    np.testing.assert_array_equal(vc[untouched], vc0[untouched])
    np.testing.assert_allclose(abar.sum(axis=1), 1.0, atol=1e-13)


# ---------------------------------------------------------------- whole step
def test_select_all_equals_full_recomputation():
    """k >= |M|, p = 1, one block: every step must reproduce full recomputation."""
    wd, su = TINY, TINY_SETUP
    dims, mdl = _dims(wd), _tiny_model(1)
    y0, m0 = W.initial_sequence(wd, su, 0)
    L = su.seq_len
    prm = O.Params(sigma=su.sigma, k=L, p=1.0, block_len=su.gen_len, n_unmask=1)
    st = O.new_state(dims, y0, m0, su.prompt_len)
    for t in range(su.gen_len):
        y_in, masked_in = st.y.copy(), st.is_masked.copy()
        O.d2cache_step(dims, mdl, prm, st)
        assert list(st.trace["S"]) == list(range(L))
        full = O.full_forward(dims, mdl, y_in)
        np.testing.assert_allclose(st.trace["hidden"], full["hidden"], rtol=1e-9, atol=1e-10)
        np.testing.assert_allclose(st.k_cache, full["k"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(st.v_cache, full["v"], rtol=1e-9, atol=1e-11)
        rows = np.flatnonzero(masked_in)
        np.testing.assert_allclose(st.trace["logits"], full["logits"][rows], rtol=1e-9, atol=1e-10)
        for l in range(wd.n_layers):
            np.testing.assert_allclose(st.trace["abars"][l], full["attn_mean"][l], rtol=1e-9, atol=1e-13)
        # vanilla decoding on top of it: confidences are the full model's
        s_full, x_full = O.confidence(full["logits"][rows])
        np.testing.assert_allclose(st.conf[rows], s_full.astype(np.float32), rtol=1e-6)
        np.testing.assert_array_equal(st.pred[rows], x_full)
    assert not st.is_masked.any()


def test_select_none_leaves_cache_unchanged():
    wd = TINY
    dims, mdl = _dims(wd), _tiny_model(2)
    L = 12
    kc = W.hidden_rows(8, L, wd.d_kv).astype(np.float64)
    vc = W.hidden_rows(9, L, wd.d_kv).astype(np.float64)
    kc0, vc0 = kc.copy(), vc.copy()
    h, abar = O.refresh_layer(dims, mdl["layers"][0], np.zeros((0, wd.d_model)), np.zeros(0, np.int64), kc, vc)
    assert h.shape == (0, wd.d_model) and abar.shape == (0, L)
    assert kc.tobytes() == kc0.tobytes() and vc.tobytes() == vc0.tobytes()
    # whole step with an empty S: caches, confidences and predictions stay bit-identical
    y0, m0 = W.initial_sequence(wd, TINY_SETUP, 0)
    st = O.new_state(dims, y0, m0, TINY_SETUP.prompt_len)
    O.d2cache_step(dims, mdl, O.Params(sigma=2.0, k=3, p=0.5, block_len=5), st)
    snap = (st.k_cache.tobytes(), st.v_cache.tobytes(), st.conf.tobytes(), st.pred.tobytes())
    st.S = np.zeros(0, np.int32)
    O.d2cache_step(dims, mdl, O.Params(sigma=2.0, k=3, p=0.5, block_len=5), st)
    assert snap == (st.k_cache.tobytes(), st.v_cache.tobytes(), st.conf.tobytes(), st.pred.tobytes())
    np.testing.assert_array_equal(st.trace["c"], np.ones(TINY_SETUP.seq_len))     # S = {} => c = 1


@pytest.mark.parametrize("seed", range(3))
def test_step_brute_force_tiny(seed):
    """L = 8, V = 16, one layer: the whole step as scalar nested sums."""
    wd = W.ModelDims(1, 8, 2, 1, 4, 12, 16, dtype="f32")
    su = W.DecodeSetup(3, 5, 3, 1, k=2, p=0.4, sigma=1.5)
    dims, mdl = _dims(wd), _tiny_model(seed, wd, std_scale=20.0)
    y0, m0 = W.initial_sequence(wd, su, seed)
    prm = O.Params(sigma=su.sigma, k=su.k, p=su.p, block_len=su.block_len, n_unmask=su.n_unmask)
    st = O.new_state(dims, y0, m0, su.prompt_len)
    bs = None
    for t in range(su.gen_len):
        before = dict(y=st.y.copy(), is_masked=st.is_masked.copy(), k=st.k_cache[0].copy(), v=st.v_cache[0].copy(),
                      conf=st.conf.copy(), pred=st.pred.copy(), S=st.S.copy())
        O.d2cache_step(dims, mdl, prm, st)
        ref = brute_step(wd, mdl, prm, su.prompt_len, before)
        np.testing.assert_allclose(st.k_cache[0], ref["k"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(st.v_cache[0], ref["v"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(st.trace["hidden"], ref["hidden"], rtol=1e-9, atol=1e-10)
        np.testing.assert_allclose(st.trace["c"], ref["c"], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(st.trace["D"], ref["D"], rtol=1e-12)
        np.testing.assert_allclose(st.conf, ref["conf"], rtol=1e-6)
        np.testing.assert_array_equal(st.pred, ref["pred"])
        assert list(st.trace["mstar"]) == ref["mstar"]
        assert list(st.trace["decode"]) == ref["decode"]
        assert list(st.trace["u"]) == ref["u"]
        assert list(st.S) == ref["s_next"]
        np.testing.assert_array_equal(st.y, ref["y"])
        np.testing.assert_array_equal(st.is_masked, ref["is_masked"])
    assert not st.is_masked.any()


@pytest.mark.parametrize("seed", range(2))
def test_step_rollout_over_first_layers(seed):
    """The lightweight rollout of the appendix (rollout over the first r layers only): on a 4-layer model
    the influence scores of d2cache_step(rollout_layers = r) must equal Eq. 6-9 written as nested loops over
    the step's own head-averaged attention of layers 0 .. r-1 (not the last r, not r +- 1), r = N must equal
    r = 0 (all layers), and r = 1 must equal the single-layer closed form
    c_j = [j not in S] + sum_{i in S} (A_ij + [i = j]) / 2.  The forward pass itself does not depend on r."""
    wd = W.ModelDims(4, 16, 2, 1, 8, 24, 32, dtype="f32")
    su = W.DecodeSetup(5, 7, 4, 1, k=2, p=0.4, sigma=1.5)
    dims, mdl = _dims(wd), _tiny_model(seed + 5, wd, std_scale=12.0)
    y0, m0 = W.initial_sequence(wd, su, seed)
    L, N = su.seq_len, wd.n_layers
    traces = {}
    for r in (0, 1, 2, 3, N, N + 3):
        prm = O.Params(sigma=su.sigma, k=su.k, p=su.p, block_len=su.block_len, n_unmask=1, rollout_layers=r)
        st = O.new_state(dims, y0, m0, su.prompt_len)
        O.d2cache_step(dims, mdl, prm, st)                       # step 0: every row
        first = dict(st.trace)
        # the second step from a FIXED partial row set, so that every r sees the same S
        st.S = np.array([1, 4, 6, 7, 10], np.int32)
        O.d2cache_step(dims, mdl, prm, st)
        traces[r] = (first, dict(st.trace))
    for r, steps in traces.items():
        for tr in steps:
            S, abars = tr["S"], tr["abars"]
            assert len(abars) == N
            used = abars if r == 0 else abars[:min(r, N)]
            np.testing.assert_allclose(tr["c"], brute_influence(used, S, L), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(tr["c"], O.influence(O.rollout(used, S, L)), rtol=0, atol=0)
            assert abs(tr["c"].sum() - L) < 1e-11
    for step in (0, 1):
        base = traces[0][step]
        for r in traces:
            for l in range(N):                                   # the forward does not depend on r
                np.testing.assert_array_equal(traces[r][step]["abars"][l], base["abars"][l])
        np.testing.assert_array_equal(traces[N][step]["c"], base["c"])
        np.testing.assert_array_equal(traces[N + 3][step]["c"], base["c"])
        # r = 1: the closed form of one layer, from layer 0's attention (and not from the last layer's)
        tr = traces[1][step]
        S, a0, a_last = [int(i) for i in tr["S"]], tr["abars"][0], tr["abars"][-1]
        for j in range(L):
            ref = (0.0 if j in S else 1.0) + sum(0.5 * (a0[q, j] + (1.0 if S[q] == j else 0.0)) for q in range(len(S)))
            assert abs(tr["c"][j] - ref) < 1e-13
        wrong = np.array([(0.0 if j in S else 1.0) + sum(0.5 * (a_last[q, j] + (1.0 if S[q] == j else 0.0))
                                                         for q in range(len(S))) for j in range(L)])
        assert np.max(np.abs(wrong - tr["c"])) > 1e-3            # the pin can tell the first layer from the last
        # and the depths differ from one another, so an off-by-one would show
        cs = [traces[r][step]["c"] for r in (1, 2, 3, N)]
        for a, b in zip(cs, cs[1:]):
            assert np.max(np.abs(a - b)) > 1e-4


def test_generation_loop_contract():
    """Sec. 3.1: one token leaves M per step, blocks finish left to right,
    decoded tokens are never re-masked, and S_{t+1} holds the token just decoded."""
    wd, su = W.DIMS["C1"], W.SETUP["C1"]
    small = W.with_layers(wd, 1)
    dims = _dims(small)
    mdl = W.model_weights(small, 0)
    y0, m0 = W.initial_sequence(small, su, 0)
    prm = O.Params(sigma=su.sigma, k=su.k, p=su.p, block_len=su.block_len, n_unmask=su.n_unmask)
    seen = []

    def on_step(t, st):
        dec = st.trace["decode"]
        assert len(dec) == 1 and set(dec) <= set(st.trace["mstar"])
        assert set(dec) <= set(st.S)                                   # R3
        lo, hi = st.trace["block"]
        assert lo == su.prompt_len + (t // su.block_len) * su.block_len
        assert lo <= dec[0] < hi
        assert len(st.trace["mstar"]) == min(su.k, su.block_len - t % su.block_len)
        assert st.y[dec[0]] == st.pred[dec[0]]
        seen.append(int(dec[0]))

    st = O.generate(dims, mdl, prm, y0, m0, su.prompt_len, on_step=on_step)
    assert sorted(seen) == list(range(su.prompt_len, su.seq_len))
    assert not st.is_masked.any()
