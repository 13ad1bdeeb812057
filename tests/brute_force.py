"""Scalar, token-at-a-time reference used only to pin the CPU oracle on tiny inputs.

Pure Python floats and lists, no numpy, no matrix products, nothing shared with
`oracle/`.  Tokens are processed one at a time the way a decoder generates them:
token t of a layer reads the cache rows 0..t that earlier tokens left behind.
Under causal attention this equals a batched prefill, which is what the oracle
does; agreement between the two therefore checks the oracle's masks, head
grouping, rotary pairing, residual wiring and cache indexing.
"""
import math


def _matvec(w, x):                      # w: [out][in]
    return [sum(wi * xi for wi, xi in zip(row, x)) for row in w]


def _rms(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [v * r * gi for v, gi in zip(x, g)]


def _rot(vec, angle_pos, base):
    dh = len(vec)
    half = dh // 2
    out = [0.0] * dh
    for i in range(half):
        ang = angle_pos * base ** (-2.0 * i / dh)
        c, s = math.cos(ang), math.sin(ang)
        out[i] = vec[i] * c - vec[i + half] * s
        out[i + half] = vec[i + half] * c + vec[i] * s
    return out


class TinyModel:
    def __init__(self, m):
        """m: anything with the oracle model's attribute names; weights become nested lists."""
        self.L, self.d, self.hq, self.hkv, self.dh = m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim
        self.base, self.eps = float(m.rope_base), float(m.rms_eps)
        self.layers = [{k: [[float(v) for v in row] for row in w[k]] if w[k].ndim == 2 else [float(v) for v in w[k]]
                        for k in w} for w in m.layers]
        self.g_final = [float(v) for v in m.g_final]
        self.w_lm = [[float(v) for v in row] for row in m.w_lm]


def token_layer(tm, l, h, pos, kc, vc):
    """Run one token (hidden h at position pos) through layer l; kc/vc: dict pos -> [Hkv][dh]."""
    w = tm.layers[l]
    a = _rms(h, w["g_attn"], tm.eps)
    q = _matvec(w["wq"], a)
    k = _matvec(w["wk"], a)
    v = _matvec(w["wv"], a)
    dh = tm.dh
    kc[pos] = [_rot(k[j * dh:(j + 1) * dh], pos, tm.base) for j in range(tm.hkv)]
    vc[pos] = [v[j * dh:(j + 1) * dh] for j in range(tm.hkv)]
    return q


def token_attend(tm, l, h, q, pos, kc, vc):
    w = tm.layers[l]
    dh, g = tm.dh, tm.hq // tm.hkv
    o = []
    for i in range(tm.hq):
        qi = _rot(q[i * dh:(i + 1) * dh], pos, tm.base)
        keys = [t for t in sorted(kc) if t <= pos]
        sc = [sum(a * b for a, b in zip(qi, kc[t][i // g])) / math.sqrt(dh) for t in keys]
        mx = max(sc)
        e = [math.exp(v - mx) for v in sc]
        z = sum(e)
        for c in range(dh):
            o.append(sum(e[n] / z * vc[t][i // g][c] for n, t in enumerate(keys)))
    h = [a + b for a, b in zip(h, _matvec(w["wo"], o))]
    f = _rms(h, w["g_ffn"], tm.eps)
    gate = _matvec(w["w_gate"], f)
    up = _matvec(w["w_up"], f)
    act = [gv / (1.0 + math.exp(-gv)) * uv for gv, uv in zip(gate, up)]
    return [a + b for a, b in zip(h, _matvec(w["w_down"], act))]


def brute_full_prefill(tm, x):
    """Token-by-token forward of x (list of [d] lists).  Returns (kc, vc, h_in, logits):
    kc[l][pos] -> [Hkv][dh]; h_in[l][t] is the hidden state entering layer l."""
    T = len(x)
    kc = [dict() for _ in range(tm.L)]
    vc = [dict() for _ in range(tm.L)]
    h_in = [[None] * T for _ in range(tm.L + 1)]
    for t in range(T):                       # one token at a time, all layers
        h = list(x[t])
        for l in range(tm.L):
            h_in[l][t] = h
            q = token_layer(tm, l, h, t, kc[l], vc[l])
            h = token_attend(tm, l, h, q, t, kc[l], vc[l])
        h_in[tm.L][t] = h
    logits = _matvec(tm.w_lm, _rms(h_in[tm.L][T - 1], tm.g_final, tm.eps))
    return kc, vc, h_in, logits


def brute_relay(tm, x_prefix, k_src_pre, v_src, h_start, l_start, l_det, l_end, k):
    """Selective-recompute prefill with scalar loops (no suffix, pre-RoPE keys).

    k_src_pre / v_src: [L][S][Hkv][dh] nested lists; h_start: [S][d].
    Returns (kc, vc, sel, score, logits).
    """
    P, S = len(x_prefix), len(h_start)
    kc = [dict() for _ in range(tm.L)]
    vc = [dict() for _ in range(tm.L)]
    for l in range(tm.L):
        for j in range(S):
            kc[l][P + j] = [_rot(k_src_pre[l][j][hh], P + j, tm.base) for hh in range(tm.hkv)]
            vc[l][P + j] = [list(v_src[l][j][hh]) for hh in range(tm.hkv)]
    hid = {t: list(x_prefix[t]) for t in range(P)}          # position -> hidden, for active rows
    sel, score = [], None
    for l in range(tm.L):
        if l == l_start:
            if k > 0:
                for j in range(S):
                    hid[P + j] = list(h_start[j])
            else:
                hid[P + S - 1] = list(h_start[S - 1])
        if l == l_det and k > 0:
            w = tm.layers[l]
            score = []
            for j in range(S):
                vf = _matvec(w["wv"], _rms(hid[P + j], w["g_attn"], tm.eps))
                acc = 0.0
                for hh in range(tm.hkv):
                    a = vc[l][P + j][hh]
                    b = vf[hh * tm.dh:(hh + 1) * tm.dh]
                    dot = sum(u * v for u, v in zip(a, b))
                    na = math.sqrt(sum(u * u for u in a))
                    nb = math.sqrt(sum(v * v for v in b))
                    acc += dot / max(na * nb, 1e-12)
                score.append(1.0 - acc / tm.hkv)
            ranked = sorted(range(S), key=lambda j: (-score[j], j))
            sel = sorted(ranked[:k])
            keep = set(sel) | {S - 1}
            for j in range(S):
                if j not in keep:
                    del hid[P + j]
        if l == l_end + 1:
            for t in list(hid):
                if P <= t < P + S - 1:
                    del hid[t]
        active = sorted(hid)
        qs = {t: token_layer(tm, l, hid[t], t, kc[l], vc[l]) for t in active}     # write K/V first
        hid = {t: token_attend(tm, l, hid[t], qs[t], t, kc[l], vc[l]) for t in active}
    logits = _matvec(tm.w_lm, _rms(hid[P + S - 1], tm.g_final, tm.eps))
    return kc, vc, sel, score, logits


def brute_decode_influence(tm, x, n_prompt):
    """Feed x[0..T) one token at a time; for the steps t >= n_prompt (the decoding steps) add every
    attention weight of the step's token, over all layers and query heads, to s_inf[key position].
    Returns (s_inf[T], logits of the last step)."""
    T = len(x)
    kc = [dict() for _ in range(tm.L)]
    vc = [dict() for _ in range(tm.L)]
    s_inf = [0.0] * T
    h = None
    dh, g = tm.dh, tm.hq // tm.hkv
    for t in range(T):
        h = list(x[t])
        for l in range(tm.L):
            q = token_layer(tm, l, h, t, kc[l], vc[l])
            if t >= n_prompt:
                for i in range(tm.hq):
                    qi = _rot(q[i * dh:(i + 1) * dh], t, tm.base)
                    sc = [sum(a * b for a, b in zip(qi, kc[l][j][i // g])) / math.sqrt(dh) for j in range(t + 1)]
                    mx = max(sc)
                    z = sum(math.exp(v - mx) for v in sc)
                    for j in range(t + 1):
                        s_inf[j] += math.exp(sc[j] - mx) / z
            h = token_attend(tm, l, h, q, t, kc[l], vc[l])
    return s_inf, _matvec(tm.w_lm, _rms(h, tm.g_final, tm.eps))


def brute_relay_multi(tm, pieces, l_start, l_det, l_end):
    """Scalar single-pass prefill of a prompt made of ("new", x) and ("seg", k_pre, v, h_start, k) pieces
    (nested lists).  The prompt ends with new text.  Returns (kc, vc, sels, logits)."""
    kc = [dict() for _ in range(tm.L)]
    vc = [dict() for _ in range(tm.L)]
    hid, segs, t = {}, [], 0
    for pc in pieces:
        if pc[0] == "new":
            for row in pc[1]:
                hid[t] = list(row)
                t += 1
        else:
            _, k_pre, v, h_start, k = pc
            n = len(h_start)
            for l in range(tm.L):
                for j in range(n):
                    kc[l][t + j] = [_rot(k_pre[l][j][hh], t + j, tm.base) for hh in range(tm.hkv)]
                    vc[l][t + j] = [list(v[l][j][hh]) for hh in range(tm.hkv)]
            segs.append((t, n, h_start, k))
            t += n
    sels = [[] for _ in segs]
    for l in range(tm.L):
        if l == l_start:
            for p0, n, h_start, k in segs:
                if k > 0:
                    for j in range(n):
                        hid[p0 + j] = list(h_start[j])
        if l == l_det:
            w = tm.layers[l]
            for si, (p0, n, h_start, k) in enumerate(segs):
                if k <= 0:
                    continue
                score = []
                for j in range(n):
                    vf = _matvec(w["wv"], _rms(hid[p0 + j], w["g_attn"], tm.eps))
                    acc = 0.0
                    for hh in range(tm.hkv):
                        a, b = vc[l][p0 + j][hh], vf[hh * tm.dh:(hh + 1) * tm.dh]
                        dot = sum(u * v for u, v in zip(a, b))
                        acc += dot / max(math.sqrt(sum(u * u for u in a)) * math.sqrt(sum(v * v for v in b)), 1e-12)
                    score.append(1.0 - acc / tm.hkv)
                ranked = sorted(range(n), key=lambda j: (-score[j], j))
                sels[si] = sorted(ranked[:k])
                for j in range(n):
                    if j not in sels[si]:
                        del hid[p0 + j]
        if l == l_end + 1:
            for p0, n, _, _ in segs:
                for j in range(n):
                    hid.pop(p0 + j, None)
        active = sorted(hid)
        qs = {p: token_layer(tm, l, hid[p], p, kc[l], vc[l]) for p in active}
        hid = {p: token_attend(tm, l, hid[p], qs[p], p, kc[l], vc[l]) for p in active}
    logits = _matvec(tm.w_lm, _rms(hid[t - 1], tm.g_final, tm.eps))
    return kc, vc, sels, logits
