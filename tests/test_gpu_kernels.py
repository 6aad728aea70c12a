"""GPU parity of the individual C-ABI calls against the CPU oracle:
d2c_attention, d2c_refresh_layer, d2c_influence, d2c_select.  Same seeded inputs on
both sides; floats within rel-L2 1e-5 (fp32) / 2e-2 (bf16), index sets bit-exact."""
import numpy as np
import pytest
import torch

from oracle import d2cache_oracle as O
from paper_2509_23094_amd import workloads as W

from gpu_util import TOL, host, oracle_dims, rel_l2, say, topk_margin

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2509_23094_amd import binding
    return binding


def _ctx_for(B, wd, max_seq, n_layers=1, seed=0, tiny_vocab=None, tunables=None):
    dims = W.with_layers(wd, n_layers)
    if tiny_vocab is not None:
        from dataclasses import replace
        dims = replace(dims, vocab=tiny_vocab)
    mdl = W.model_weights(dims, seed)
    return B.Context(dims, mdl, max_seq, tunables=tunables), dims, mdl


# ------------------------------------------------------------------ the ragged-row projection
LINEAR_CASES = [
    # dtype, m, N, K
    ("f32", 1, 16, 16), ("f32", 72, 768, 256), ("f32", 128, 1376, 256), ("f32", 37, 256, 688), ("f32", 5, 40, 20),
    ("f32", 200, 100, 132),
    ("bf16", 1, 64, 128), ("bf16", 83, 1024, 512), ("bf16", 17, 40, 72), ("bf16", 96, 4096, 1408),
    ("bf16", 130, 200, 264), ("bf16", 300, 3000, 520), ("bf16", 64, 33000, 256),
    ("bf16", 185, 1000, 392), ("bf16", 192, 4096, 512), ("bf16", 200, 520, 256),   # 12 row tiles in one chunk; two chunks
]


@pytest.mark.parametrize("dtype,m,N,K", LINEAR_CASES)
def test_linear_parity(B, dtype, m, N, K, tunables=None):
    say(f"linear dtype={dtype} m={m} N={N} K={K} tunables={tunables}")
    wd = W.ModelDims(1, 256, 4, 4, 64, 80, 64, dtype=dtype)
    ctx, _, _ = _ctx_for(B, wd, max_seq=max(m, 16), tunables=tunables)
    a = W.hidden_rows(11, m, K)
    w = W.hidden_rows(12, N, K, std=0.05)
    if dtype == "bf16":
        a, w = W.round_bf16(a), W.round_bf16(w)
    out = torch.full((m, N), 7.0, dtype=torch.float32, device="cuda")
    ctx.d2c_linear(B.to_device(a, dtype), B.to_device(w, dtype), m, N, K, out)
    torch.cuda.synchronize()
    ref = a.astype(np.float64) @ w.astype(np.float64).T          # exact inputs on both sides: fp32 accumulation only
    assert rel_l2(host(out), ref) < 1e-5
    ctx.close()


@pytest.mark.parametrize("waves", [4, 6, 7, 8, 10])
@pytest.mark.parametrize("dtype,m,N,K", [("f32", 37, 250, 132), ("bf16", 70, 1000, 520), ("bf16", 9, 176, 4096)])
def test_linear_parity_every_workgroup_width(B, waves, dtype, m, N, K):
    """The planner picks 6, 8 or 10 waves per workgroup by shape; here each width (and the 4-wave one) is
    forced on shapes whose column count is no multiple of the workgroup's columns."""
    test_linear_parity(B, dtype, m, N, K, tunables={"gemm_waves": waves})


# ------------------------------------------------------------------ attention (config "C2" and edge shapes)
ATTN_CASES = [
    # dtype, H, Hkv, dh, L, m, kernels ("few": the few-row kernels, "tiled": the LDS-tiled ones, "default":
    # the library's own choice, "": fp32)
    ("bf16", 32, 32, 128, 2048, 256, "tiled"),    # the isolated selective-refresh attention workload, full size
    ("bf16", 32, 32, 128, 2048, 256, "few"),
    ("bf16", 28, 4, 128, 768, 83, "few"),         # Dream geometry (GQA 28/4), ragged m
    ("bf16", 28, 4, 128, 768, 83, "tiled"),       # two query tiles per wave, split key range, ragged last block
    ("bf16", 4, 2, 64, 203, 37, "few"),           # head_dim 64, ragged L and m
    ("bf16", 4, 2, 64, 203, 37, "tiled"),
    ("bf16", 8, 8, 128, 17, 1, "few"),            # one query, L smaller than a workgroup's key span
    ("bf16", 8, 8, 128, 17, 1, "tiled"),          # a single, mostly empty key block
    ("bf16", 4, 4, 128, 130, 130, "few"),         # every row selected
    ("bf16", 4, 4, 128, 130, 130, "tiled"),
    ("bf16", 32, 32, 128, 3072, 300, "tiled"),    # long-context shape: no key split, 3 query blocks, 48 key blocks
    ("bf16", 3, 1, 64, 1000, 129, "tiled"),       # odd head count (A-bar loop tail), head_dim 64, 3 query blocks
    ("bf16", 6, 3, 64, 100, 20, "few"),           # 3 kv heads: neither divides nor is divided by the 8 XCDs
    ("bf16", 16, 2, 128, 600, 50, "few"),         # 4 XCDs per kv head, 8 query heads each; L above 512
    ("bf16", 32, 32, 128, 512, 46, "few"),        # the LLaDA-8B decode step: 96 (tile, head) pairs
    ("bf16", 5, 5, 128, 300, 16, "few"),          # 5 kv heads: plain placement
    ("bf16", 28, 4, 128, 1824, 93, "default"),    # the long-generation decode step late on: too long for the
                                                  # per-head probability rows, so the tiled kernels from 48 rows on
    ("bf16", 28, 4, 128, 1824, 40, "default"),    # same length, fewer rows: few-row kernels and their second launch
    ("f32", 4, 4, 64, 128, 73, ""),               # the small fp32 model's geometry
    ("f32", 4, 2, 8, 19, 5, ""),
]


@pytest.mark.parametrize("dtype,H,Hkv,dh,L,m,kernels", ATTN_CASES)
def test_attention_parity(B, dtype, H, Hkv, dh, L, m, kernels):
    say(f"attention dtype={dtype} H={H} Hkv={Hkv} dh={dh} L={L} m={m} kernels={kernels}")
    tun = {"attn_tiled_min_m": 1 if kernels == "tiled" else 1 << 30} if kernels in ("tiled", "few") else None
    _attention_parity(B, dtype, H, Hkv, dh, L, m, tunables=tun)


def test_attention_short_sequence_in_a_long_context(B):
    """A context sized for 2048 positions serving L = 256: the short sequence is split into more head groups
    and key ranges than the longest one, so the scratch buffers must be sized over every L, not max_seq."""
    say("attention L=256 m=200 in a max_seq=2048 context")
    _attention_parity(B, "bf16", 8, 8, 128, 256, 200, max_seq=2048, tunables={"attn_tiled_min_m": 1})


def _attention_parity(B, dtype, H, Hkv, dh, L, m, max_seq=None, tunables=None):
    wd = W.ModelDims(1, H * dh, H, Hkv, dh, 64, 64, dtype=dtype)
    ctx, dims, _ = _ctx_for(B, wd, max_seq=max_seq or L, tunables=tunables)
    case = W.attention_case(1, H, Hkv, dh, L, m, dtype=dtype)
    tdt = B.torch_dtype(dtype)
    q = B.to_device(case["q"], dtype)
    kc, vc = B.to_device(case["k_cache"], dtype), B.to_device(case["v_cache"], dtype)
    nk, nv = B.to_device(case["new_k"], dtype), B.to_device(case["new_v"], dtype)
    idx = torch.from_numpy(case["idx"]).cuda()
    out = torch.zeros((m, H * dh), dtype=tdt, device="cuda")
    abar = torch.zeros((m, L), dtype=torch.float32, device="cuda")
    ctx.d2c_attention(q, idx, m, nk, nv, kc, vc, L, out, abar)
    torch.cuda.synchronize()

    k_ref, v_ref = case["k_cache"].astype(np.float64), case["v_cache"].astype(np.float64)
    k_ref[case["idx"]] = case["new_k"]
    v_ref[case["idx"]] = case["new_v"]
    # the scatter is a copy: bit-exact
    np.testing.assert_array_equal(host(kc), k_ref.astype(np.float32))
    np.testing.assert_array_equal(host(vc), v_ref.astype(np.float32))
    o_ref, a_ref = O.selective_attention(case["q"], k_ref, v_ref, H, Hkv, dh)
    og, ag = host(out), host(abar)
    for r in range(m):
        assert rel_l2(og[r], o_ref[r]) < TOL[dtype], f"output row {r}"
        assert rel_l2(ag[r], a_ref[r]) < TOL[dtype], f"A-bar row {r}"
    np.testing.assert_allclose(host(abar).sum(axis=1), 1.0, atol=2e-3 if dtype == "bf16" else 1e-5)

    # without the head average the output must not change; run-to-run the bits must not change
    out2 = torch.zeros_like(out)
    ctx.d2c_attention(q, idx, m, None, None, kc, vc, L, out2, None)
    abar3, out3 = torch.zeros_like(abar), torch.zeros_like(out)
    ctx.d2c_attention(q, idx, m, None, None, kc, vc, L, out3, abar3)
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(out, out3) and torch.equal(abar, abar3)
    ctx.close()


# ------------------------------------------------------------------ one block on the selected rows
LAYER_CASES = [
    # name, dims, L, m, tolerance-scale
    ("C1-f32", W.DIMS["C1"], 128, 72),
    ("C1-f32-all", W.DIMS["C1"], 128, 128),
    ("tiny-f32-gqa", W.ModelDims(1, 64, 4, 2, 16, 80, 64, dtype="f32"), 33, 7),
    ("bf16-small", W.ModelDims(1, 512, 4, 4, 128, 1408, 64, dtype="bf16"), 200, 45),
    ("bf16-gqa", W.ModelDims(1, 512, 8, 2, 64, 1024, 64, dtype="bf16"), 300, 150),
    ("bf16-185-rows", W.ModelDims(1, 512, 4, 4, 128, 1408, 64, dtype="bf16"), 260, 185),   # 12 row tiles in one chunk
    ("C3-width", W.DIMS["C3"], 512, 83),     # one LLaDA-8B-shaped layer at full width
    ("C4-width", W.DIMS["C4"], 768, 100),    # one Dream-7B-shaped layer at full width
    # more than 256 rows: 128 x 64 outputs per wave in every projection (all widths are whole chunk pairs)
    ("bf16-330-rows", W.ModelDims(1, 512, 4, 4, 128, 1536, 64, dtype="bf16"), 400, 330),
    ("tiny-f32-odd-ffn", W.ModelDims(1, 64, 4, 4, 16, 72, 64, dtype="f32"), 40, 9),   # FFN width not a multiple of 16
]
# the same block with the caller's row-major weights (no pre-tiled copies, separate SwiGLU launch)
LAYER_CASES_ROW_MAJOR = ["C1-f32", "bf16-small", "C3-width"]


@pytest.mark.parametrize("name,wd,L,m", LAYER_CASES, ids=[c[0] for c in LAYER_CASES])
def test_refresh_layer_parity(B, name, wd, L, m):
    _refresh_layer_parity(B, name, wd, L, m)


@pytest.mark.parametrize("name", LAYER_CASES_ROW_MAJOR)
def test_refresh_layer_parity_row_major_weights(B, name):
    case = [c for c in LAYER_CASES if c[0] == name][0]
    _refresh_layer_parity(B, *case, tunables={"gemm_preshuffle": 0})


@pytest.mark.parametrize("waves", [6, 7, 10])
@pytest.mark.parametrize("name", ["C1-f32", "bf16-small", "tiny-f32-odd-ffn"])
def test_refresh_layer_parity_forced_workgroup_width(B, name, waves):
    """The gated epilogue pairs neighbouring waves: checked for the 6- and 10-wave workgroups on shapes where
    the planner would not pick them by itself."""
    case = [c for c in LAYER_CASES if c[0] == name][0]
    _refresh_layer_parity(B, *case, tunables={"gemm_waves": waves})


@pytest.mark.parametrize("mt", [6, 7, 8])
def test_refresh_layer_parity_forced_rows_per_workgroup(B, mt):
    """Many rows: 6, 7 or 8 row tiles per workgroup of the wide projection shape, whatever the planner's choice."""
    case = [c for c in LAYER_CASES if c[0] == "bf16-330-rows"][0]
    _refresh_layer_parity(B, *case, tunables={"gemm_wide_mt": mt})


def _refresh_layer_parity(B, name, wd, L, m, tunables=None):
    say(f"refresh_layer {name} L={L} m={m} tunables={tunables}")
    ctx, dims, mdl = _ctx_for(B, wd, max_seq=L, tiny_vocab=64, tunables=tunables)
    od = oracle_dims(dims)
    dtype = dims.dtype
    S = W.distinct_sorted_rows(3, L, m)
    h0 = W.hidden_rows(4, m, dims.d_model, std=0.5)
    kc0 = W.hidden_rows(5, L, dims.d_kv, std=1.0, extra=1)
    vc0 = W.hidden_rows(5, L, dims.d_kv, std=1.0, extra=2)
    if dtype == "bf16":
        kc0, vc0 = W.round_bf16(kc0), W.round_bf16(vc0)
    roll0 = np.abs(W.hidden_rows(6, m, L)).astype(np.float32)           # an arbitrary incoming block for layer > 0

    hidden = torch.from_numpy(h0).cuda()
    kc, vc = B.to_device(kc0, dtype), B.to_device(vc0, dtype)
    idx = torch.from_numpy(S).cuda()
    abar = torch.zeros((m, L), dtype=torch.float32, device="cuda")
    roll = torch.from_numpy(roll0).cuda()
    ctx.d2c_refresh_layer(0, hidden, idx, S, kc, vc, L, abar, roll)
    torch.cuda.synchronize()

    k_ref, v_ref = kc0.astype(np.float64), vc0.astype(np.float64)
    h_ref, a_ref = O.refresh_layer(od, mdl["layers"][0], h0, S, k_ref, v_ref)
    tol = TOL[dtype]
    # row by row: one wrong row must not hide in a norm over the whole tensor
    for r in range(m):
        assert rel_l2(host(hidden)[r], h_ref[r]) < tol, f"hidden row {r}"
        assert rel_l2(host(abar)[r], a_ref[r]) < tol, f"A-bar row {r}"
    kg, vg = host(kc), host(vc)
    for i in S:
        assert rel_l2(kg[i], k_ref[i]) < tol and rel_l2(vg[i], v_ref[i]) < tol, f"K/V row {i}"
    rest = np.setdiff1d(np.arange(L), S)
    np.testing.assert_array_equal(host(kc)[rest], kc0[rest])             # reused rows: untouched bits
    np.testing.assert_array_equal(host(vc)[rest], vc0[rest])
    # layer 0 starts the rollout from the identity: C_S = (A-bar + one-hot) / 2
    c_ref = O.rollout([a_ref], S, L)[S]
    assert rel_l2(host(roll), c_ref) < tol
    ctx.close()


def test_refresh_layer_rollout_chain_and_influence(B):
    """Three layers in a row on the same rows: the compact rollout block and c_j against the literal L x L rollout."""
    wd = W.ModelDims(3, 256, 4, 4, 64, 688, 64, dtype="f32")
    L, m = 96, 29
    say(f"rollout chain L={L} m={m}")
    mdl = W.model_weights(wd, 2)
    ctx = B.Context(wd, mdl, L)
    od = oracle_dims(wd)
    S = W.distinct_sorted_rows(7, L, m)
    h0 = W.hidden_rows(8, m, wd.d_model, std=0.5)
    hidden = torch.from_numpy(h0).cuda()
    idx = torch.from_numpy(S).cuda()
    kcs = [W.hidden_rows(9, L, wd.d_kv, extra=l) for l in range(3)]
    vcs = [W.hidden_rows(10, L, wd.d_kv, extra=l) for l in range(3)]
    roll = torch.zeros((m, L), dtype=torch.float32, device="cuda")
    abar = torch.zeros((m, L), dtype=torch.float32, device="cuda")
    h_ref, abars = h0.astype(np.float64), []
    for l in range(3):
        kc, vc = B.to_device(kcs[l], "f32"), B.to_device(vcs[l], "f32")
        ctx.d2c_refresh_layer(l, hidden, idx, S, kc, vc, L, abar, roll)
        h_ref, a = O.refresh_layer(od, mdl["layers"][l], h_ref, S, kcs[l].astype(np.float64), vcs[l].astype(np.float64))
        abars.append(a)
    infl = torch.zeros(L, dtype=torch.float32, device="cuda")
    ctx.d2c_influence(roll, idx, m, L, infl)
    torch.cuda.synchronize()
    C = O.rollout(abars, S, L)
    assert rel_l2(host(hidden), h_ref) < 1e-5
    assert rel_l2(host(roll), C[S]) < 1e-5
    assert rel_l2(host(infl), O.influence(C)) < 1e-5
    assert abs(float(host(infl).sum()) - L) < 1e-3
    ctx.close()


def test_refresh_layer_empty_and_errors(B):
    wd = W.ModelDims(1, 64, 4, 2, 16, 80, 64, dtype="f32")
    L = 20
    ctx, dims, _ = _ctx_for(B, wd, max_seq=L)
    say("refresh_layer m=0 and argument errors")
    hidden = torch.ones((4, 64), device="cuda")
    kc = torch.randn((L, dims.d_kv), device="cuda")
    vc = torch.randn((L, dims.d_kv), device="cuda")
    kc0, vc0, h0 = kc.clone(), vc.clone(), hidden.clone()
    idx = torch.tensor([1, 5, 6, 9], dtype=torch.int32, device="cuda")
    empty = np.zeros(0, np.int32)
    ctx.d2c_refresh_layer(0, hidden, idx, empty, kc, vc, L, None, None)                # m = 0: nothing touched
    torch.cuda.synchronize()
    assert torch.equal(kc, kc0) and torch.equal(vc, vc0) and torch.equal(hidden, h0)
    for bad in ([5, 1, 6, 9], [1, 5, 5, 9], [1, 5, 6, 20], [-1, 5, 6, 9]):
        with pytest.raises(B.D2CError) as ei:
            ctx.d2c_refresh_layer(0, hidden, idx, np.array(bad, np.int32), kc, vc, L, None, None)
        assert ei.value.code == B.D2C_EINVAL
    with pytest.raises(B.D2CError) as ei:
        ctx.d2c_refresh_layer(0, hidden, idx, np.array([1, 5, 6, 9], np.int32), kc, vc, L + 1, None, None)
    assert ei.value.code == B.D2C_ESHAPE
    with pytest.raises(B.D2CError) as ei:
        ctx.d2c_refresh_layer(3, hidden, idx, np.array([1, 5, 6, 9], np.int32), kc, vc, L, None, None)
    assert ei.value.code == B.D2C_EINVAL
    torch.cuda.synchronize()
    assert torch.equal(kc, kc0) and torch.equal(vc, vc0) and torch.equal(hidden, h0)   # nothing written on error
    ctx.close()


# ------------------------------------------------------------------ selection
def _run_select(B, ctx, prm, logits, logit_pos, y, is_masked, P, conf, pred, c):
    L = len(y)
    dev = "cuda"
    t = {
        "tokens": torch.from_numpy(y.astype(np.int32)).to(dev), "is_masked": torch.from_numpy(is_masked.astype(np.uint8)).to(dev),
        "conf": torch.from_numpy(conf.astype(np.float32)).to(dev), "pred": torch.from_numpy(pred.astype(np.int32)).to(dev),
        "influence": torch.from_numpy(c.astype(np.float32)).to(dev),
    }
    for name in ("mstar", "u_set", "decode_idx", "s_next", "s_rows_next"):
        t[name] = torch.full((L,), -1, dtype=torch.int32, device=dev)
    t["counts"] = torch.zeros(B.N_COUNTS, dtype=torch.int32, device=dev)
    t["score"] = torch.zeros(L, dtype=torch.float32, device=dev)
    lg = torch.from_numpy(logits).to(dev) if len(logit_pos) else None
    lp = torch.from_numpy(logit_pos.astype(np.int32)).to(dev) if len(logit_pos) else None
    ctx.d2c_select(prm, lg, lp, len(logit_pos), t["tokens"], t["is_masked"], L, P, t["conf"], t["pred"], t["influence"],
                   t["mstar"], t["u_set"], t["decode_idx"], t["s_next"], t["s_rows_next"], t["counts"], t["score"])
    torch.cuda.synchronize()
    cnt = t["counts"].cpu().numpy()
    res = {k: v.cpu().numpy() for k, v in t.items()}
    res["mstar"] = res["mstar"][: cnt[B.CNT_MSTAR]]
    res["u_set"] = res["u_set"][: cnt[B.CNT_U]]
    res["decode_idx"] = res["decode_idx"][: cnt[B.CNT_DECODE]]
    res["s_next"] = res["s_next"][: cnt[B.CNT_S]]
    res["s_rows_next"] = res["s_rows_next"][: cnt[B.CNT_NEXT_ROWS]]
    return res, cnt


SELECT_CASES = [
    # L, P, vocab, block_len, k, n_unmask, p, sigma, frac_known, cand_mode, skewed[, threshold, conf_decode]
    (128, 64, 1024, 32, 8, 1, 0.9, 10.0, 0.0, 0, False),
    (128, 64, 1024, 32, 8, 1, 0.9, 10.0, 0.4, 0, True),
    (512, 256, 126464, 32, 32, 1, 0.1, 10.0, 0.3, 0, True),      # LLaDA-8B-shaped step, full vocabulary
    (768, 512, 152064, 32, 32, 1, 0.1, 10.0, 0.6, 0, False),     # Dream-7B-shaped
    (3072, 2048, 4096, 64, 32, 2, 0.1, 10.0, 0.5, 0, True),      # long context
    (3072, 2048, 4096, 1024, 32, 2, 0.1, 40.0, 0.5, 0, True),    # fully non-autoregressive: one block
    (333, 100, 777, 50, 7, 3, 0.35, 3.0, 0.5, 1, True),          # ragged everything, literal candidate mode
    (64, 8, 64, 16, 100, 100, 1.0, 10.0, 0.2, 0, False),         # select-all switch, unmask the whole block
    (40, 40, 64, 8, 4, 1, 0.5, 10.0, 0.0, 0, False),             # nothing masked
    (97, 0, 64, 32, 5, 1, 0.0, 10.0, 0.1, 0, True),              # no prompt, p = 0
    (512, 256, 4096, 32, 8, 1, 0.1, 10.0, 0.3, 0, True, 0.5, 0),     # parallel decoding: threshold on s^i
    (512, 256, 4096, 32, 8, 2, 0.1, 10.0, 0.3, 0, True, 0.0, 1),     # decode by confidence alone
    (300, 100, 512, 64, 4, 1, 0.2, 5.0, 0.5, 1, False, 0.9, 1),      # both, literal candidate mode
]


@pytest.mark.parametrize("case", SELECT_CASES, ids=[str(i) for i in range(len(SELECT_CASES))])
def test_select_parity(B, case):
    L, P, V, blk, k, nu, p, sigma, frac, mode, skew = case[:11]
    thr, cdec = (case[11], case[12]) if len(case) > 11 else (0.0, 0)
    say(f"select L={L} P={P} V={V} block={blk} k={k} n_unmask={nu} p={p} sigma={sigma} mode={mode} thr={thr} cdec={cdec}")
    wd = W.ModelDims(1, 64, 4, 4, 16, 80, V, dtype="f32")
    mdl = W.model_weights(W.ModelDims(1, 64, 4, 4, 16, 80, 8, dtype="f32"), 0)
    mdl["tok_emb"] = mdl["lm_head"] = np.zeros((V, 64), np.float32)      # the selection never touches them
    ctx = B.Context(wd, mdl, L)
    seed = L + V
    is_masked = W.random_mask(seed, L, P, frac).astype(bool) if L > P else np.zeros(L, bool)
    y = np.where(is_masked, wd.mask_id, 7).astype(np.int32)
    conf0 = W.random_scores(seed, L)
    pred0 = (np.arange(L) * 7 % V).astype(np.int32)
    c = W.skewed_influence(seed, L) if skew else (W.random_scores(seed + 1, L) + np.float32(0.5))
    c[3 % L] = c[(L // 2)] = c[L - 1]                                     # exact ties in the influence
    masked_pos = np.flatnonzero(is_masked)
    logit_pos = masked_pos[:: 3][:16]                                     # rows that were in this step's forward
    logits = W.logits_rows(seed, len(logit_pos), V) if len(logit_pos) else np.zeros((0, V), np.float32)
    if len(logit_pos) > 1:
        logits[1, 5] = logits[1, 2] = logits[1].max() + 1.0               # tied maxima: lowest index wins
    prm = B.make_params(sigma, k, p, blk, nu, mode, thr, cdec)
    res, cnt = _run_select(B, ctx, prm, logits, logit_pos, y, is_masked, P, conf0, pred0, c)

    # Eq. 1
    conf_ref, pred_ref = conf0.astype(np.float64), pred0.copy()
    if len(logit_pos):
        s, xh = O.confidence(logits)
        conf_ref[logit_pos], pred_ref[logit_pos] = s, xh
    np.testing.assert_array_equal(res["pred"], pred_ref)
    np.testing.assert_allclose(res["conf"], conf_ref, rtol=1e-5)
    # Eq. 3: scores within tolerance
    oprm = O.Params(sigma=sigma, k=k, p=p, block_len=blk, n_unmask=nu, cand_mode=mode, threshold=thr, conf_decode=cdec)
    sel = O.select(oprm, is_masked, P, conf_ref.astype(np.float32), c)
    lo, hi = sel["block"]
    cand1 = np.array([i for i in range(lo, hi) if is_masked[i]], np.int64)
    assert (cnt[B.CNT_BLOCK_LO], cnt[B.CNT_BLOCK_HI]) == (lo, hi)
    if len(cand1):
        np.testing.assert_allclose(res["score"][cand1], sel["score"][cand1], rtol=1e-5)
    # Eq. 4 and the decode set: integer-exact on the score array the GPU itself produced
    np.testing.assert_array_equal(res["mstar"], O.top_k_select(res["score"], cand1, k))
    dec_ref = O.top_k_select(res["conf"] if cdec else res["score"], cand1, nu)      # on the GPU's own float arrays
    if thr > 0:
        dec_ref = np.union1d(dec_ref, cand1[res["conf"][cand1] > np.float32(thr)]).astype(np.int32)
    np.testing.assert_array_equal(res["decode_idx"], dec_ref)
    if topk_margin(sel["score"], cand1, k) > 1e-4:
        np.testing.assert_array_equal(res["mstar"], sel["mstar"])
    conf_margin = np.min(np.abs(conf_ref[cand1] - thr) / max(thr, 1e-9)) if thr > 0 and len(cand1) else 1.0
    if topk_margin(conf_ref if cdec else sel["score"], cand1, nu) > 1e-4 and conf_margin > 1e-4:
        np.testing.assert_array_equal(res["decode_idx"], sel["decode"])
    # stage 2 is decided on the given float32 influence array: bit-exact always
    cand2 = np.flatnonzero(~is_masked) if mode == 0 else np.setdiff1d(np.arange(L), res["mstar"])
    np.testing.assert_array_equal(res["u_set"], O.top_p_select(c, cand2, p))
    np.testing.assert_array_equal(res["s_next"], np.union1d(np.union1d(res["mstar"], res["decode_idx"]), res["u_set"]))
    # Eq. 2
    y_ref, m_ref = y.copy(), is_masked.copy()
    y_ref[res["decode_idx"]] = pred_ref[res["decode_idx"]]
    m_ref[res["decode_idx"]] = False
    np.testing.assert_array_equal(res["tokens"], y_ref)
    np.testing.assert_array_equal(res["is_masked"].astype(bool), m_ref)
    np.testing.assert_array_equal(res["s_rows_next"], np.flatnonzero(m_ref[res["s_next"]]))
    assert cnt[B.CNT_MASKED] == int(m_ref.sum())
    ctx.close()


def test_select_large_equal_scores_and_errors(B):
    """All scores equal: top-k takes the lowest indices, top-p the first floor(p n)+1 known tokens."""
    L, P, V = 256, 100, 64
    say("select equal scores")
    wd = W.ModelDims(1, 64, 4, 4, 16, 80, V, dtype="f32")
    mdl = W.model_weights(wd, 0)
    ctx = B.Context(wd, mdl, L)
    is_masked = np.zeros(L, bool); is_masked[P:] = True
    y = np.where(is_masked, wd.mask_id, 3).astype(np.int32)
    # conf chosen so that D * conf is the same float for every candidate is impossible in general (D varies);
    # sigma huge makes D constant instead
    conf = np.full(L, 0.25, np.float32)
    c = np.ones(L, np.float32)
    prm = B.make_params(1e6, 5, 0.25, L, 2, 0)
    res, cnt = _run_select(B, ctx, prm, np.zeros((0, V), np.float32), np.zeros(0, np.int32), y, is_masked, P, conf,
                           np.zeros(L, np.int32), c)
    assert list(res["mstar"]) == [P, P + 1, P + 2, P + 3, P + 4]
    assert list(res["decode_idx"]) == [P, P + 1]
    assert list(res["u_set"]) == list(range(int(0.25 * P) + 1))
    for bad in (dict(sigma=0.0), dict(k=-1), dict(block_len=0), dict(p=-0.5), dict(cand_mode=2), dict(threshold=-1.0),
                dict(conf_decode=3), dict(rollout_layers=-2)):
        kw = dict(sigma=10.0, k=4, p=0.1, block_len=32, n_unmask=1, cand_mode=0)
        kw.update(bad)
        with pytest.raises(B.D2CError) as ei:
            _run_select(B, ctx, B.make_params(**kw), np.zeros((0, V), np.float32), np.zeros(0, np.int32), y, is_masked,
                        P, conf, np.zeros(L, np.int32), c)
        assert ei.value.code == B.D2C_EINVAL
    ctx.close()


@pytest.mark.parametrize("P,blk,inside", [(20, 8, 17), (20, 8, 3), (5, 8, 2)])
def test_select_masked_position_inside_prompt(B, P, blk, inside):
    """A masked position before the end of the prompt (legal input, not produced by the decoding loop): blocks
    are counted from the prompt's end in both directions, so the current block is the one holding it."""
    L, V = 64, 64
    say(f"select with a masked prompt position P={P} block={blk} inside={inside}")
    wd = W.ModelDims(1, 64, 4, 4, 16, 80, V, dtype="f32")
    ctx = B.Context(wd, W.model_weights(wd, 0), L)
    is_masked = np.zeros(L, bool)
    is_masked[[inside, inside + 1, 40, 41]] = True
    y = np.where(is_masked, wd.mask_id, 3).astype(np.int32)
    conf = W.random_scores(P, L)
    c = W.random_scores(P + 1, L) + np.float32(0.5)
    res, cnt = _run_select(B, ctx, B.make_params(3.0, 1, 0.2, blk, 1, 0), np.zeros((0, V), np.float32),
                           np.zeros(0, np.int32), y, is_masked, P, conf, np.zeros(L, np.int32), c)
    sel = O.select(O.Params(sigma=3.0, k=1, p=0.2, block_len=blk, n_unmask=1), is_masked, P, conf, c)
    assert (cnt[B.CNT_BLOCK_LO], cnt[B.CNT_BLOCK_HI]) == sel["block"]
    lo, hi = sel["block"]
    assert lo <= inside < hi
    cand1 = np.array([i for i in range(lo, hi) if is_masked[i]], np.int64)
    np.testing.assert_array_equal(res["mstar"], O.top_k_select(res["score"], cand1, 1))
    np.testing.assert_array_equal(res["decode_idx"], O.top_k_select(res["score"], cand1, 1))
    np.testing.assert_array_equal(res["u_set"], sel["u"])
    ctx.close()


def test_tunables_belong_to_a_context(B):
    """Two live contexts with different tunables give the launch shapes each asked for, a live context can be
    re-tuned, and the pre-tiled weight copies can only be chosen at init."""
    say("per-context tunables")
    wd = W.ModelDims(1, 256, 4, 4, 64, 80, 64, dtype="bf16")
    mdl = W.model_weights(wd, 0)
    ctx_a = B.Context(wd, mdl, 64, tunables={"gemm_waves": 4, "gemm_max_splits": 1})
    ctx_b = B.Context(wd, mdl, 64)
    m, N, K = 40, 1000, 520
    a = W.round_bf16(W.hidden_rows(11, m, K))
    w = W.round_bf16(W.hidden_rows(12, N, K, std=0.05))
    ref = a.astype(np.float64) @ w.astype(np.float64).T
    outs = []
    for ctx in (ctx_a, ctx_b, ctx_a):
        out = torch.zeros((m, N), dtype=torch.float32, device="cuda")
        ctx.d2c_linear(B.to_device(a, "bf16"), B.to_device(w, "bf16"), m, N, K, out)
        torch.cuda.synchronize()
        assert rel_l2(host(out), ref) < 1e-5
        outs.append(out)
    assert torch.equal(outs[0], outs[2])                       # context a is unaffected by what b ran in between
    ctx_b.set_tunable("gemm_waves", 10)
    out = torch.zeros((m, N), dtype=torch.float32, device="cuda")
    ctx_b.d2c_linear(B.to_device(a, "bf16"), B.to_device(w, "bf16"), m, N, K, out)
    torch.cuda.synchronize()
    assert rel_l2(host(out), ref) < 1e-5
    with pytest.raises(B.D2CError) as ei:
        ctx_b.set_tunable("gemm_preshuffle", 0)
    assert ei.value.code == B.D2C_EINVAL
    with pytest.raises(B.D2CError) as ei:
        ctx_b.set_tunable("no_such_knob", 1)
    assert ei.value.code == B.D2C_EINVAL
    info = ctx_a.memory_info()
    assert info["total_bytes"] == ctx_a.workspace_bytes() and 0 < info["pretiled_weight_bytes"] < info["total_bytes"]
    ctx_a.close()
    ctx_b.close()
