"""Benchmark of the d2Cache selective-refresh decoding step on one MI355X.

Workload: the LLaDA-8B-shaped random-init model (32 layers, d_model 4096, 32x128
heads, SwiGLU 12288, vocabulary 126464, bf16), prompt 256 + 256 generated
positions, blocks of 32, one token unmasked per step, sigma 10 / k 32 / p 0.1.
A "step" is one d2c_step: partial forward of the selected rows through all 32
layers with rollout, LM head + Eq. 1 on the masked rows, two-stage selection and
unmasking.  Step 0 (all 512 rows) fills the caches before the clock starts.

Prints one JSON line.  value = timed steps / wall time between two device synchronisations;
roofline = algorithmic weight bytes of the projection launches / their HIP-event durations
(a second pass over the same steps with an event pair around every launch), against 8 TB/s;
full_recompute = the same engine with every row selected; generation = one whole generation timed
from before step 0 to the last token (generated tokens per second); cpu_baseline = the CPU oracle on a
bounded sample of the same workload.  --workload C4 / C5 / C6 / C2 / select / parallel run the other
configurations; memory = device bytes the library holds beside the caller's buffers.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0        # dense bf16 matrix-core peak of the chip


def device_model(W, dims, seed, torch):
    """Random-init weights N(0, 0.02) drawn on the device (seeded), in the storage type."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    tdt = torch.bfloat16 if dims.dtype == "bf16" else torch.float32

    def normal(*shape):
        t = torch.empty(shape, dtype=torch.float32, device="cuda")
        t.normal_(0.0, 0.02, generator=g)
        return t.to(tdt).contiguous()

    ones = lambda n: torch.ones(n, dtype=torch.float32, device="cuda")
    d, dq, dkv, f = dims.d_model, dims.d_q, dims.d_kv, dims.d_ffn
    layers = []
    for _ in range(dims.n_layers):
        layers.append({"attn_norm": ones(d), "wqkv": normal(dq + 2 * dkv, d), "wo": normal(d, dq),
                       "ffn_norm": ones(d), "w_gate_up": normal(2 * f, d), "w_down": normal(d, f)})
    return {"tok_emb": normal(dims.vocab, d), "final_norm": ones(d), "lm_head": normal(dims.vocab, d),
            "layers": layers}


def fresh_sequences(B, W, ctx, dims, su, gen):
    """One batch of independent sequences (different prompts, same lengths)."""
    seqs = []
    for b in range(su.batch):
        y0, m0 = W.initial_sequence(dims, su, gen * su.batch + b)
        seqs.append(B.Sequence_(ctx, y0, m0, su.prompt_len))
    return seqs


def cpu_baseline(W, dims, su, m_rows, n_logit_rows, n_steps=2):
    """The oracle on this machine's host cores, on a bounded sample of the same workload: n_steps whole d2Cache
    steps at the mean shapes of the timed run (m_rows selected rows, n_logit_rows masked rows), each step =
    n_layers x (one full-width block on the selected rows + its L x L rollout update) + LM head + Eq. 1 +
    both selections.  The weights of one layer are reused for every layer (the cost is the same per
    layer; 16 GB of fp32 weights per layer set would not fit the sample's time), nothing is scaled."""
    import numpy as np
    from oracle import d2cache_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    od = O.Dims(1, dims.d_model, dims.n_heads, dims.n_kv_heads, dims.head_dim, dims.d_ffn, dims.vocab,
                dims.rms_eps, dims.rope_theta)
    L = su.seq_len
    lw = W.layer_weights(dims, 0, 0)
    head = {"final_norm": np.ones(dims.d_model), "lm_head": W.lm_head(dims, 0)}
    S = W.distinct_sorted_rows(0, L, m_rows)
    h0 = W.hidden_rows(0, m_rows, dims.d_model, std=0.5)
    kc = W.round_bf16(W.hidden_rows(1, L, dims.d_kv)).astype(np.float64)
    vc = W.round_bf16(W.hidden_rows(2, L, dims.d_kv)).astype(np.float64)
    is_masked = W.random_mask(0, L, su.prompt_len, 0.3).astype(bool)
    conf = W.random_scores(0, L)
    prm = O.Params(sigma=su.sigma, k=su.k, p=su.p, block_len=su.block_len, n_unmask=su.n_unmask)
    t_layers = t_roll = t_head = t_sel = 0.0
    t_all = time.perf_counter()
    for _ in range(n_steps):
        h, abars = h0, []
        t0 = time.perf_counter()
        for _l in range(dims.n_layers):
            h, abar = O.refresh_layer(od, lw, h, S, kc, vc)
            abars.append(abar)
            h = h0                                    # the same, well-scaled input for every layer
        t_layers += time.perf_counter() - t0
        t0 = time.perf_counter()
        C = O.rollout(abars, S, L)
        t_roll += time.perf_counter() - t0
        t0 = time.perf_counter()
        s, xh = O.confidence(O.lm_logits(od, head, h[:n_logit_rows]))
        t_head += time.perf_counter() - t0
        t0 = time.perf_counter()
        O.select(prm, is_masked, su.prompt_len, conf, O.influence(C).astype(np.float32))
        t_sel += time.perf_counter() - t0
    total = time.perf_counter() - t_all
    return {"value": n_steps / total, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": ("%d whole steps at the run's mean shapes (%d selected rows, %d masked rows, L = %d), %.1f s: "
                       "%d x (full-width block + rollout update) with one layer's weights reused %.1f s + %.1f s, "
                       "LM head + Eq. 1 %.1f s, selection %.2f s"
                       % (n_steps, m_rows, n_logit_rows, L, total, dims.n_layers, t_layers, t_roll, t_head, t_sel))}


def bench_select_op(args, B, W, torch, np):
    """The isolated two-stage selection (Eq. 1, 3, 4, top-p over the influence scores) at the two sequence
    lengths of the step workloads, on two input regimes: weakly structured scores (what random-init weights
    give) and skewed ones (a few sink positions carry most of the influence, a Zipf-like tail, and a few
    confident rows), which is what trained models show.  Latency-bound: reported in microseconds per call."""
    # every call decodes one token in place, so the masked set shrinks by one per call: the repetitions are
    # capped well below the ~180 masked positions the inputs start with
    K, Wm = min(args.steps, 64), min(args.warmup, 8)
    res = {}
    for L, P, V, k, n_rows in ((512, 256, 126464, 32, 32), (3072, 2048, 126464, 32, 32)):
        wd = W.ModelDims(1, 64, 4, 4, 16, 80, V, dtype="f32")
        mdl = W.model_weights(W.ModelDims(1, 64, 4, 4, 16, 80, 8, dtype="f32"), 0)
        mdl["tok_emb"] = mdl["lm_head"] = np.zeros((V, 64), np.float32)      # the selection never reads them
        ctx = B.Context(wd, mdl, L)
        prm = B.make_params(10.0, k, 0.1, 32, 1, 0)
        is_masked = W.random_mask(L, L, P, 0.3).astype(bool)
        y = np.where(is_masked, wd.mask_id, 7).astype(np.int32)
        masked_pos = np.flatnonzero(is_masked)
        logit_pos = masked_pos[:n_rows].astype(np.int32)
        logits = W.logits_rows(L, len(logit_pos), V)
        for regime in ("weak", "skewed"):
            if regime == "weak":
                conf, c = W.random_scores(L, L), W.random_scores(L + 1, L) + np.float32(0.5)
            else:
                conf = (W.random_scores(L, L) ** 8).astype(np.float32)
                c = W.skewed_influence(L, L)
            t = {"tokens": torch.from_numpy(y).cuda(), "is_masked": torch.from_numpy(is_masked.astype(np.uint8)).cuda(),
                 "conf": torch.from_numpy(conf.astype(np.float32)).cuda(),
                 "pred": torch.zeros(L, dtype=torch.int32, device="cuda"),
                 "influence": torch.from_numpy(c.astype(np.float32)).cuda(),
                 "counts": torch.zeros(B.N_COUNTS, dtype=torch.int32, device="cuda"),
                 "score": torch.zeros(L, dtype=torch.float32, device="cuda")}
            for name in ("mstar", "u_set", "decode_idx", "s_next", "s_rows_next"):
                t[name] = torch.full((L,), -1, dtype=torch.int32, device="cuda")
            lg, lp = torch.from_numpy(logits).cuda(), torch.from_numpy(logit_pos).cuda()

            def call():
                ctx.d2c_select(prm, lg, lp, len(logit_pos), t["tokens"], t["is_masked"], L, P, t["conf"], t["pred"],
                               t["influence"], t["mstar"], t["u_set"], t["decode_idx"], t["s_next"], t["s_rows_next"],
                               t["counts"], t["score"])
            for _ in range(Wm):
                call()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(K):
                call()
            e1.record()
            torch.cuda.synchronize()
            cnt = t["counts"].cpu().numpy()
            res["L%d_%s" % (L, regime)] = {"us_per_call": round(1e3 * e0.elapsed_time(e1) / K, 2),
                                           "n_mstar": int(cnt[B.CNT_MSTAR]), "n_u": int(cnt[B.CNT_U]),
                                           "logit_rows": int(len(logit_pos)), "vocab": V}
        ctx.close()
    main_r = res["L512_skewed"]
    logits_bytes = 32 * 126464 * 4
    return {
        "metric": "selection_calls_per_sec", "value": round(1e6 / main_r["us_per_call"], 1), "unit": "calls/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(main_r["us_per_call"] / 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "isolated d2c_select: 32 logit rows x vocab 126464, L 512 (and 3072), sigma 10, k 32, "
                               "p 0.1; weakly structured and skewed confidence / influence inputs"},
        "roofline": {"bound": "hbm", "achieved": round(logits_bytes / main_r["us_per_call"] / 1e3, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(logits_bytes / main_r["us_per_call"] / 1e3 / HBM_PEAK_GBS, 4), "traffic": None,
                     "note": "latency-bound chain of three small launches; the only streamed bytes are the logits"},
        "variants": res, "cpu_baseline": None,
    }


def bench_attention_op(args, B, W, torch, np, tune=None):
    """The isolated selective-refresh attention op: scatter of m new K/V rows, then m queries against all
    L cached keys, no mask, with and without the head-averaged probabilities.  One "step" = one call."""
    H, Hkv, dh, L, m = 32, 32, 128, 2048, 256
    wd = W.with_layers(W.ModelDims(1, H * dh, H, Hkv, dh, 64, 64, dtype="bf16"), 1)
    ctx = B.Context(wd, W.model_weights(wd, 0), L, tunables=tune)
    case = W.attention_case(1, H, Hkv, dh, L, m, dtype="bf16")
    q = B.to_device(case["q"], "bf16")
    kc, vc = B.to_device(case["k_cache"], "bf16"), B.to_device(case["v_cache"], "bf16")
    nk, nv = B.to_device(case["new_k"], "bf16"), B.to_device(case["new_v"], "bf16")
    idx = torch.from_numpy(case["idx"]).cuda()
    out = torch.zeros((m, H * dh), dtype=torch.bfloat16, device="cuda")
    abar = torch.zeros((m, L), dtype=torch.float32, device="cuda")
    K, Wm = args.steps, args.warmup
    flops = 4.0 * H * m * L * dh
    # K, V once; Q, O; scatter reads and writes 2 m d_kv; A-bar write when asked for
    base_bytes = 2 * (2 * L * Hkv * dh) + 2 * (2 * m * H * dh) + 2 * 2 * (2 * m * Hkv * dh)
    res = {}
    for name, ab in (("with_head_average", abar), ("output_only", None)):
        for _ in range(Wm):
            ctx.d2c_attention(q, idx, m, nk, nv, kc, vc, L, out, ab)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(K):
            ctx.d2c_attention(q, idx, m, nk, nv, kc, vc, L, out, ab)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        us = 1e3 * e0.elapsed_time(e1) / K
        by = base_bytes + (4 * m * L if ab is not None else 0)
        # the head average comes out of the forward pass (unnormalised probabilities kept per key block): no extra flops
        res[name] = {"us_per_call": round(us, 2), "wall_us_per_call": round(1e6 * wall / K, 2),
                     "tflops": round(flops / us / 1e6, 1), "mfma_frac": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "gbs": round(by / us / 1e3, 1), "hbm_frac": round(by / us / 1e3 / HBM_PEAK_GBS, 4)}
    ctx.close()
    main_r = res["with_head_average"]
    return {
        "metric": "selective_attention_calls_per_sec", "value": round(1e6 / main_r["us_per_call"], 1), "unit": "calls/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(main_r["us_per_call"] / 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C2: isolated selective-refresh attention, 32 heads x 128, L 2048, m 256 query rows, "
                               "scatter of 256 new K/V rows, no mask"},
        "roofline": {"bound": "mfma", "achieved": main_r["tflops"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": main_r["mfma_frac"], "traffic": None, "flops_per_call": flops,
                     "hbm_frac": main_r["hbm_frac"], "bytes_per_call": base_bytes + 4 * m * L},
        "variants": res, "cpu_baseline": None,
    }


def bench_parallel_decoding(args, B, W, torch, np, tune=None):
    """Whole generations at the LLaDA-8B shape with parallel decoding (appendix, parallel decoding settings):
    besides the best-scored token every stage-1 candidate whose confidence exceeds 0.9 is unmasked in the same
    step, so a generation takes fewer steps than tokens.  Random-init weights give near-uniform predictions
    (confidence ~1e-4), so the LM-head weights are scaled up until the confidences spread around the threshold;
    the timed quantity is generated tokens per second, step 0 included (the paper's throughput definition)."""
    dims, su = W.DIMS["C3"], W.SETUP["C3"]
    if args.layers:
        dims = W.with_layers(dims, args.layers)
    mdl = device_model(W, dims, 0, torch)
    mdl["lm_head"] = (mdl["lm_head"].float() * args.head_scale).to(mdl["lm_head"].dtype).contiguous()
    ctx = B.Context(dims, mdl, su.seq_len, device_weights=True, max_batch=1, tunables=tune)
    out = {}
    for name, thr in (("threshold_0.9", 0.9), ("one_token_per_step", 0.0)):
        prm = B.make_params(su.sigma, su.k, su.p, su.block_len, su.n_unmask, 0, threshold=thr,
                            rollout_layers=args.rollout_layers)
        n_gen = 1 + max(1, min(4, args.steps // 64))               # the first generation is the warm-up
        tokens = steps = 0
        elapsed = 0.0
        for gidx in range(n_gen):
            seqs = fresh_sequences(B, W, ctx, dims, su, gidx)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n = 0
            while seqs[0].n_masked > 0 and n < 4 * su.gen_len:
                ctx.d2c_step(prm, seqs)
                n += 1
            torch.cuda.synchronize()
            if gidx > 0:
                elapsed += time.perf_counter() - t0
                tokens += su.gen_len - seqs[0].n_masked
                steps += n
        out[name] = {"tokens_per_sec": round(tokens / elapsed, 2), "tokens_per_step": round(tokens / steps, 3),
                     "steps": steps, "tokens": tokens, "ms_per_step": round(1e3 * elapsed / steps, 4),
                     "generations": n_gen - 1}
    ctx.close()
    main_r = out["threshold_0.9"]
    return {
        "metric": "generated_tokens_per_sec", "value": main_r["tokens_per_sec"], "unit": "tokens/s", "n_gpus": 1,
        "steps": main_r["steps"], "warmup": 1, "ms_per_step": main_r["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dims.dtype, "data": "synthetic",
        "config": {"workload": "parallel decoding at the C3 shape (LLaDA-8B geometry, prompt %d + gen %d, block %d): "
                               "confidence threshold 0.9, LM-head weights x %g, whole generations incl. step 0"
                               % (su.prompt_len, su.gen_len, su.block_len, args.head_scale)},
        "variants": out, "speedup_over_one_token_per_step": round(main_r["tokens_per_sec"] /
                                                                    out["one_token_per_step"]["tokens_per_sec"], 3),
        "roofline": None, "cpu_baseline": None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C3", choices=["C3", "C4", "C5", "C6", "C2", "select", "parallel"],
                    help="C3 (default, the metric's workload), C4, C5, C6 (other model shapes / lengths), C2 = the isolated "
                         "selective-refresh attention op, select = the isolated selection, parallel = whole generations "
                         "at the C3 shape with parallel decoding by confidence threshold 0.9")
    ap.add_argument("--head-scale", type=float, default=12.0,
                    help="parallel workload: factor on the random LM-head weights, so that the confidences of a "
                         "random-init model spread around the threshold")
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers (the result is then not the metric)")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="library tunable of the context (include/d2c_tools.h), e.g. --tune gemm_target_wgs=768")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run five plain 256 MiB device copies (known size, for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE) and exit")
    ap.add_argument("--rollout-layers", type=int, default=0,
                    help="attention rollout over the first R layers only (the paper's lightweight variant, "
                         "R = 5 there); 0 = all layers, the metric's setting")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-vanilla", action="store_true")
    ap.add_argument("--no-generation", action="store_true", help="skip the whole-generation leg (tokens/s incl. step 0)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (sequences are independent, so "
              "the path would shard by sequence with replicated weights and no exchange)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2509_23094_amd import binding as B
    from paper_2509_23094_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tune = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in args.tune}
    if args.copy_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.zeros_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 256 << 20, "copies": 5}))
        return
    if args.workload == "C2":
        print(json.dumps(bench_attention_op(args, B, W, torch, np, tune)))
        return
    if args.workload == "select":
        print(json.dumps(bench_select_op(args, B, W, torch, np)))
        return
    if args.workload == "parallel":
        print(json.dumps(bench_parallel_decoding(args, B, W, torch, np, tune)))
        return
    dims, su = W.DIMS[args.workload], W.SETUP[args.workload]
    if args.layers:
        dims = W.with_layers(dims, args.layers)
    K, Wm = args.steps, args.warmup
    per_gen = su.gen_len // su.n_unmask - 1              # d2Cache steps one generation offers after step 0
    assert Wm < per_gen, "warmup must be shorter than one generation"

    mdl = device_model(W, dims, 0, torch)
    ctx = B.Context(dims, mdl, su.seq_len, device_weights=True, max_batch=su.batch, tunables=tune)
    prm = B.make_params(su.sigma, su.k, su.p, su.block_len, su.n_unmask, 0, rollout_layers=args.rollout_layers)

    def run_steps(seqs, n, collect=None):
        for _ in range(n):
            if collect is not None:
                collect.append((sum(q.n_s for q in seqs), sum(q.n_rows for q in seqs)))
            ctx.d2c_step(prm, seqs)

    # ---- timed region: exactly K d2Cache steps (in as many generations as needed), after W warm-up steps
    elapsed, done, shapes, gen = 0.0, 0, [], 0
    while done < K:
        seq = fresh_sequences(B, W, ctx, dims, su, gen)
        run_steps(seq, 1)                                 # step 0: every row, fills the caches (not timed)
        run_steps(seq, Wm if gen == 0 else 0)             # warm-up
        n = min(K - done, per_gen - (Wm if gen == 0 else 0))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(seq, n, shapes)
        torch.cuda.synchronize()
        elapsed += time.perf_counter() - t0
        done += n
        gen += 1
    ms_per_step = 1e3 * elapsed / K
    mean_m = float(np.mean([s[0] for s in shapes]))
    mean_rows = float(np.mean([s[1] for s in shapes]))

    # ---- roofline pass: the same steps again with an event pair around every launch
    seq = fresh_sequences(B, W, ctx, dims, su, 0)
    run_steps(seq, 1 + Wm)
    n_prof = min(K, per_gen - Wm)
    torch.cuda.synchronize()
    ctx.d2c_profile_begin()
    run_steps(seq, n_prof)
    prof = ctx.d2c_profile_end()
    gm = prof["gemm"]
    gemm_ms = gm["ms"] / max(1, gm["launches"])
    gemm_gbs = gm["bytes"] / max(1e-12, gm["ms"] * 1e-3) / 1e9
    # measured HBM bytes per projection launch (rocprofv3 counters, profiles/gemm_rows_traffic.*): the stored
    # figure describes the default workload's decode steps only, so it is reported for that workload only
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_rows_traffic.json")
    if os.path.exists(tpath) and not args.layers and not tune and args.rollout_layers == 0:
        try:
            tj = json.load(open(tpath))
            if str(tj.get("workload", "")).split()[0] == args.workload:
                traffic = tj.get("hbm_bytes_per_launch")
        except Exception:
            traffic = None
    roofline = {"bound": "hbm", "kernel": "gemm_rows_kernel", "achieved": round(gemm_gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(gemm_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                "avg_launch_us": round(1e3 * gemm_ms, 2), "launches_per_step": gm["launches"] / n_prof,
                "bytes_per_launch": gm["bytes"] / max(1, gm["launches"]),
                "measured": "HIP events around every projection launch, repeat of the timed steps"}
    by_class = {k: {"ms_per_step": round(v["ms"] / n_prof, 4), "launches_per_step": v["launches"] / n_prof}
                for k, v in prof.items()}
    step_bytes = gm["bytes"] / n_prof + prof["attention"]["bytes"] / n_prof

    # ---- full recomputation (the paper's Vanilla): the same engine with every row selected
    vanilla = None
    if not args.no_vanilla:
        seqv = fresh_sequences(B, W, ctx, dims, su, 0)
        # k >= |M|, p = 1 and a single block select every row at every step
        pv = B.make_params(su.sigma, su.seq_len, 1.0, su.gen_len, su.n_unmask, 0)
        for _ in range(2):
            ctx.d2c_step(pv, seqv)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nv = 4
        for _ in range(nv):
            assert all(q.n_s == su.seq_len for q in seqv)
            ctx.d2c_step(pv, seqv)
        torch.cuda.synchronize()
        vanilla = {"ms_per_step": round(1e3 * (time.perf_counter() - t0) / nv, 3), "rows_per_step": su.seq_len * su.batch}
        vanilla["steps_per_sec"] = round(1e3 / vanilla["ms_per_step"], 2)

    # ---- one whole generation, step 0 (every row, fills the caches) included: generated tokens per second
    generation = None
    if not args.no_generation:
        seqg = fresh_sequences(B, W, ctx, dims, su, 1000)
        n_gen_steps = su.gen_len // su.n_unmask
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_gen_steps):
            ctx.d2c_step(prm, seqg)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        left = sum(q.n_masked for q in seqg)
        generation = {"tokens_per_sec": round((su.batch * su.gen_len - left) / dt, 2), "seconds": round(dt, 4),
                      "steps": n_gen_steps, "tokens": su.batch * su.gen_len - left, "masked_left": left,
                      "includes": "step 0 over all %d rows per sequence" % su.seq_len}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(W, dims, su, int(round(mean_m)), max(1, int(round(mean_rows))))

    out = {
        "metric": "d2cache_steps_per_sec", "value": round(K / elapsed, 3), "unit": "steps/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dims.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: %s-shaped random-init model, %d layers, d_model %d, %dx%d heads, FFN %d, "
                               "vocab %d; prompt %d + gen %d, block %d, %d token/step, sigma %g k %d p %g"
                               % (args.workload, {"C3": "LLaDA-8B", "C4": "Dream-7B", "C5": "LLaDA-8B", "C6": "Dream-7B"}[args.workload], dims.n_layers, dims.d_model, dims.n_heads, dims.head_dim, dims.d_ffn,
                                  dims.vocab, su.prompt_len, su.gen_len, su.block_len, su.n_unmask, su.sigma, su.k,
                                  su.p),
                   "batch": su.batch, "seq_len": su.seq_len, "mean_rows_per_step": round(mean_m, 2),
                   "mean_logit_rows_per_step": round(mean_rows, 2)},
        "tokens_per_sec": round(su.batch * su.n_unmask * K / elapsed, 3),
        "algorithmic_gb_per_step": round(step_bytes / 1e9, 3),
        "step_hbm_frac": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "generation": generation,
        "memory": dict(ctx.memory_info(), note="device bytes the library holds beside the caller's weights and "
                       "K/V caches: pre-tiled copies of the projection matrices, every layer's head-averaged "
                       "attention for the rollout chain (max_batch x layers x max_seq^2 floats), attention partials"),
        "roofline": roofline, "kernel_classes": by_class, "full_recompute": vanilla, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
