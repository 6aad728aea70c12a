"""One d2Cache step of a ONE-layer model as scalar nested sums (pure Python
floats, no matrices, no numpy arithmetic), for tiny sizes only.  It follows the
paper's equations term by term (Eq. 1, 3, 4, 5-9 and the top-p rule of
Sec. 4.2) and is used to pin the numpy oracle."""
import math


def _rms(vec, gain, eps):
    ms = sum(v * v for v in vec) / len(vec)
    return [v / math.sqrt(ms + eps) * g for v, g in zip(vec, gain)]


def _matvec(Wm, x):
    return [sum(float(Wm[o][i]) * x[i] for i in range(len(x))) for o in range(len(Wm))]


def _rope(vec, n_heads, dh, pos, theta):
    out = list(vec)
    half = dh // 2
    for h in range(n_heads):
        for i in range(half):
            ang = pos * theta ** (-2.0 * i / dh)
            a, b = vec[h * dh + i], vec[h * dh + half + i]
            out[h * dh + i] = a * math.cos(ang) - b * math.sin(ang)
            out[h * dh + half + i] = b * math.cos(ang) + a * math.sin(ang)
    return out


def brute_step(wd, mdl, prm, prompt_len, before):
    L = len(before["y"])
    H, Hkv, dh, d, Fd, V = wd.n_heads, wd.n_kv_heads, wd.head_dim, wd.d_model, wd.d_ffn, wd.vocab
    w = mdl["layers"][0]
    y = [int(t) for t in before["y"]]
    masked = [bool(b) for b in before["is_masked"]]
    K = [[float(v) for v in row] for row in before["k"]]
    Vc = [[float(v) for v in row] for row in before["v"]]
    conf = [float(v) for v in before["conf"]]
    pred = [int(v) for v in before["pred"]]
    S = [int(i) for i in before["S"]]
    m = len(S)

    # ---- Eq. 5: forward over the rows in S, K/V of the other rows reused
    hid = [[float(v) for v in mdl["tok_emb"][y[i]]] for i in S]
    qs = []
    for r, i in enumerate(S):
        a = _rms(hid[r], [float(g) for g in w["attn_norm"]], wd.rms_eps)
        proj = _matvec(w["wqkv"], a)
        q = _rope(proj[:H * dh], H, dh, i, wd.rope_theta)
        k = _rope(proj[H * dh:H * dh + Hkv * dh], Hkv, dh, i, wd.rope_theta)
        qs.append(q)
        K[i] = k
        Vc[i] = proj[H * dh + Hkv * dh:]
    abar = [[0.0] * L for _ in range(m)]
    for r in range(m):
        att = [0.0] * (H * dh)
        for h in range(H):
            g = h // (H // Hkv)
            sc = [sum(qs[r][h * dh + e] * K[j][g * dh + e] for e in range(dh)) / math.sqrt(dh) for j in range(L)]
            mx = max(sc)
            ex = [math.exp(v - mx) for v in sc]
            z = sum(ex)
            for j in range(L):
                pj = ex[j] / z
                abar[r][j] += pj / H
                for e in range(dh):
                    att[h * dh + e] += pj * Vc[j][g * dh + e]
        o = _matvec(w["wo"], att)
        hid[r] = [hid[r][c] + o[c] for c in range(d)]
        b = _rms(hid[r], [float(g) for g in w["ffn_norm"]], wd.rms_eps)
        gu = _matvec(w["w_gate_up"], b)
        act = [gu[f] / (1.0 + math.exp(-gu[f])) * gu[Fd + f] for f in range(Fd)]
        dn = _matvec(w["w_down"], act)
        hid[r] = [hid[r][c] + dn[c] for c in range(d)]

    # ---- Eq. 6-9 with a single layer: C = W
    c = [0.0] * L
    for i in range(L):
        row = [0.0] * L
        if i in S:
            row = list(abar[S.index(i)])
        else:
            row[i] = 1.0
        row[i] += 1.0
        tot = sum(row)
        for j in range(L):
            c[j] += row[j] / tot

    # ---- Eq. 1 on the masked rows of S
    for r, i in enumerate(S):
        if masked[i]:
            xn = _rms(hid[r], [float(g) for g in mdl["final_norm"]], wd.rms_eps)
            lg = _matvec(mdl["lm_head"], xn)
            best = max(range(V), key=lambda v: (lg[v], -v))
            z = sum(math.exp(v - lg[best]) for v in lg)
            pred[i] = best
            conf[i] = float(_f32(1.0 / z))

    # ---- Eq. 3, Eq. 4, decode set
    D = [sum(math.exp(-(i - j) ** 2 / (2.0 * prm.sigma ** 2)) for j in range(L) if not masked[j]) for i in range(L)]
    score = [_f32(D[i] * conf[i]) for i in range(L)]
    first = min(i for i in range(L) if masked[i])
    lo = prompt_len + ((first - prompt_len) // prm.block_len) * prm.block_len
    hi = min(L, lo + prm.block_len)
    cand = [i for i in range(lo, hi) if masked[i]]
    ranked = sorted(cand, key=lambda i: (-score[i], i))
    mstar = sorted(ranked[:prm.k])
    decode = sorted(ranked[:prm.n_unmask])

    # ---- stage 2: smallest prefix of the known tokens whose mass exceeds p
    known = [j for j in range(L) if not masked[j]]
    c32 = [_f32(v) for v in c]
    order = sorted(known, key=lambda j: (-c32[j], j))
    q = [int(math.floor(c32[j] * 4294967296.0)) for j in order]
    thr = math.floor(_f32(prm.p) * float(sum(q)))
    u, run = list(order), 0
    for r, qv in enumerate(q):
        run += qv
        if run > thr:
            u = order[:r + 1]
            break
    u = sorted(u)

    for i in decode:
        y[i] = pred[i]
        masked[i] = False
    return {"k": K, "v": Vc, "hidden": hid, "c": c, "D": D, "conf": conf, "pred": pred, "mstar": mstar,
            "decode": decode, "u": u, "s_next": sorted(set(mstar) | set(u)), "y": y, "is_masked": masked}


def _f32(x):
    import struct
    return struct.unpack("f", struct.pack("f", x))[0]


def brute_influence(abars, S, L):
    """Eq. 6-9 over any number of layers as scalar nested loops: E^(l) (rows in S carry the head-averaged
    attention row, every other row is one-hot), W^(l) = row-normalised E^(l) + I, C^(l) = W^(l) C^(l-1)
    from C^(0) = I, and c_j = sum_i C_ij.  abars: one [|S|][L] array per layer, in layer order."""
    S = [int(i) for i in S]
    C = [[1.0 if i == j else 0.0 for j in range(L)] for i in range(L)]
    for a in abars:
        Wm = []
        for i in range(L):
            row = [0.0] * L
            if i in S:
                r = S.index(i)
                for j in range(L):
                    row[j] = float(a[r][j])
            else:
                row[i] = 1.0
            row[i] += 1.0
            tot = sum(row)
            Wm.append([v / tot for v in row])
        C = [[sum(Wm[i][t] * C[t][j] for t in range(L)) for j in range(L)] for i in range(L)]
    return [sum(C[i][j] for i in range(L)) for j in range(L)]
