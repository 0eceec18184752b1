"""Pins of the CPU oracle against things other than itself (runs without a GPU).

Each operator of oracle/stage_oracle.py is checked against closed forms,
invariants, special cases with a textbook answer, or a literal scalar loop on
tiny inputs.  The last test plants plausible mistakes into the oracle (on the
CPU) and checks that the pins notice every one of them.
"""
import math

import numpy as np
import pytest

import synth
from oracle import stage_oracle as so

TINY = synth.StageShape("f32", 2, 16, 4, 2, 4, 12, 24)  # GQA, hd=4, F=12, V=24


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ----------------------------------------------------------------------------- formats
def test_bf16_decode_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x3DCD, 0x0000, 0x4049], dtype=np.uint16)
    want = [1.0, -2.0, 0.10009765625, 0.0, 3.140625]
    assert so.decode_values(bits).tolist() == want


def test_generator_bf16_rounds_to_nearest_even():
    f = np.array([1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8, 1.0 + 2.0**-8 + 2.0**-20, -0.3], np.float32)
    got = synth.bf16_bits_from_f32(f)
    assert got[0] == 0x3F80 and got[1] == 0x3F82 and got[2] == 0x3F81
    assert abs(so.decode_values(got[3:4])[0] + 0.3) <= 2.0**-10  # half an ulp in [0.25, 0.5)


def test_layer_block_layout_hand_computed():
    # tiny fp32 benchmark config: d=256, 4 heads x 64, F=688, 4-byte elements
    lay = so.layer_block_layout(synth.CONFIGS["tiny_f32"])
    assert lay["attn_norm"] == (0, (256,))
    assert lay["wqkv"] == (1024, (768, 256))
    assert lay["wo"] == (1024 + 786432, (256, 256))
    assert lay["ffn_norm"] == (787456 + 262144, (256,))
    assert lay["wgu"] == (1049600 + 1024, (1376, 256))
    assert lay["wd"] == (1050624 + 1409024, (256, 688))
    assert lay["__bytes__"][0] == 2459648 + 704512 == 791040 * 4
    # bf16 Llama-7B layer: 202,383,360 parameters, all sizes multiples of 256 B
    lay = so.layer_block_layout(synth.CONFIGS["llama7b"])
    assert lay["__bytes__"][0] == 202383360 * 2
    # an odd size forces padding up to the next 256-byte boundary
    odd = synth.StageShape("bf16", 1, 20, 2, 1, 4, 10, 0)
    lay = so.layer_block_layout(odd)
    assert lay["wqkv"][0] == 256 and lay["wo"][0] == 1024  # 256 + 16*20*2 = 896 -> 1024


def test_unpack_reads_what_was_placed():
    s = TINY
    lay = so.layer_block_layout(s)
    t = synth.layer_tensors(s, 3, 1)
    buf = np.zeros(lay["__bytes__"][0], np.uint8)
    for name, (off, shp) in lay.items():
        if name != "__bytes__":
            raw = t[name].view(np.uint8).reshape(-1)
            buf[off : off + raw.size] = raw
    got = so.unpack_block(s, lay, buf)
    for name in t:
        np.testing.assert_array_equal(got[name], t[name].astype(np.float64))


# ----------------------------------------------------------------------------- RMSNorm
def test_rmsnorm_closed_forms():
    x = rnd(0, 5, 64) * 3.0
    eps = 1e-5
    y = so.rmsnorm(x, np.ones(64), eps)
    ms = (x**2).mean(-1)
    np.testing.assert_allclose(np.sqrt((y**2).mean(-1)), np.sqrt(ms / (ms + eps)), rtol=1e-13)
    # hand example: x=(3,4): mean square 12.5
    y = so.rmsnorm(np.array([[3.0, 4.0]]), np.array([2.0, 0.5]), 0.0)
    np.testing.assert_allclose(y, [[2 * 3 / math.sqrt(12.5), 0.5 * 4 / math.sqrt(12.5)]], rtol=1e-15)
    # eps sits inside the square root, added to the mean of squares
    y = so.rmsnorm(np.array([[3.0, 4.0]]), np.ones(2), 3.5)
    np.testing.assert_allclose(y, [[0.75, 1.0]], rtol=1e-15)
    # scale invariance (eps=0) and constant rows
    g = rnd(1, 64)
    np.testing.assert_allclose(so.rmsnorm(7.0 * x, g, 0.0), so.rmsnorm(x, g, 0.0), rtol=1e-13)
    np.testing.assert_allclose(so.rmsnorm(np.full((1, 64), -2.5), g, 0.0), -g[None, :], rtol=1e-14)


# ----------------------------------------------------------------------------- RoPE
def test_rope_explicit_angles_and_pairing():
    p = 7
    u = np.zeros((1, 1, 4))
    u[0, 0, 0] = 1.0  # pair 0, angle = pos * 1
    np.testing.assert_allclose(so.rope(u, [p], 10000.0)[0, 0], [math.cos(p), math.sin(p), 0, 0], atol=1e-15)
    u = np.zeros((1, 1, 4))
    u[0, 0, 3] = 1.0  # second element of pair 1, angle = pos * 10000^(-2/4) = pos/100
    np.testing.assert_allclose(
        so.rope(u, [p], 10000.0)[0, 0], [0, 0, -math.sin(p / 100), math.cos(p / 100)], atol=1e-15
    )
    u = np.zeros((1, 1, 8))
    u[0, 0, 6] = 1.0  # pair 3 of 4: angle = pos * 16^(-6/8)
    a = p * 16.0 ** (-0.75)
    np.testing.assert_allclose(so.rope(u, [p], 16.0)[0, 0, 6:], [math.cos(a), math.sin(a)], atol=1e-15)


def test_rope_invariants():
    u, w = rnd(2, 6, 3, 8), rnd(3, 6, 3, 8)
    pos = np.array([0, 1, 5, 17, 300, 2303])
    r = so.rope(u, pos, 10000.0)
    np.testing.assert_array_equal(r[0], u[0])  # position 0 is the identity
    np.testing.assert_allclose(
        r[..., 0::2] ** 2 + r[..., 1::2] ** 2, u[..., 0::2] ** 2 + u[..., 1::2] ** 2, rtol=1e-12
    )
    # <rope(q,m), rope(k,n)> depends on m-n only
    d0 = (so.rope(u, pos, 1e4) * so.rope(w, pos[::-1].copy(), 1e4)).sum(-1)
    d1 = (so.rope(u, pos + 11, 1e4) * so.rope(w, pos[::-1] + 11, 1e4)).sum(-1)
    np.testing.assert_allclose(d0, d1, atol=1e-11)
    # composition
    np.testing.assert_allclose(
        so.rope(so.rope(u, pos, 1e4), 2 * pos + 1, 1e4), so.rope(u, 3 * pos + 1, 1e4), atol=1e-11
    )


# ----------------------------------------------------------------------------- attention
def attention_literal(q, k, v, pos):
    """Index-by-index definition with an explicit mask, python floats only."""
    n, hq, hd = q.shape
    hkv, ctx, _ = k.shape
    out = np.zeros((n, hq, hd))
    for r in range(n):
        for h in range(hq):
            kh = h // (hq // hkv)
            sc = []
            for j in range(ctx):
                if j > pos[r]:
                    continue
                sc.append(sum(q[r, h, e] * k[kh, j, e] for e in range(hd)) / math.sqrt(hd))
            m = max(sc)
            ex = [math.exp(a - m) for a in sc]
            z = sum(ex)
            for e in range(hd):
                out[r, h, e] = sum(ex[j] / z * v[kh, j, e] for j in range(len(sc)))
    return out


def test_attention_brute_force_tiny():
    for seed, (n, hq, hkv, hd, ctx) in enumerate([(5, 4, 2, 4, 8), (1, 2, 2, 2, 6), (8, 6, 1, 4, 8)]):
        q, k, v = rnd(seed, n, hq, hd), rnd(seed + 50, hkv, ctx, hd), rnd(seed + 90, hkv, ctx, hd)
        pos = np.arange(ctx - n, ctx)
        np.testing.assert_allclose(
            so.attention_rows(q, k, v, pos), attention_literal(q, k, v, pos), rtol=1e-12, atol=1e-14
        )


def test_attention_special_cases():
    hq, hkv, hd, ctx = 4, 2, 8, 6
    q, k, v = rnd(1, ctx, hq, hd), rnd(2, hkv, ctx, hd), rnd(3, hkv, ctx, hd)
    pos = np.arange(ctx)
    o = so.attention_rows(q, k, v, pos)
    # first row sees a single key: output is v_0 of its kv head
    np.testing.assert_allclose(o[0, 3], v[1, 0], rtol=1e-14)
    np.testing.assert_allclose(o[0, 1], v[0, 0], rtol=1e-14)
    # probabilities sum to one: constant values come back unchanged
    np.testing.assert_allclose(so.attention_rows(q, k, np.ones_like(v), pos), 1.0, rtol=1e-14)
    # all keys equal: causal running mean of the values
    keq = np.broadcast_to(k[:, :1], k.shape)
    want = np.cumsum(v, axis=1) / np.arange(1, ctx + 1)[None, :, None]
    got = so.attention_rows(q, keq, v, pos)
    for h in range(hq):
        np.testing.assert_allclose(got[:, h], want[h // 2], rtol=1e-13)
    # closed form with the 1/sqrt(hd) scale: hd=4, scores (0, 2*1/2)
    q1 = np.zeros((1, 1, 4)); q1[0, 0, 0] = 2.0
    k1 = np.zeros((1, 2, 4)); k1[0, 1, 0] = 1.0
    v1 = np.zeros((1, 2, 4)); v1[0, 0, 0] = 1.0; v1[0, 1, 1] = 1.0
    o1 = so.attention_rows(q1, k1, v1, np.array([1]))
    np.testing.assert_allclose(o1[0, 0, :2], [1 / (1 + math.e), math.e / (1 + math.e)], rtol=1e-14)
    # jointly permuting earlier keys and values leaves the last row unchanged
    perm = np.array([3, 0, 4, 2, 1, 5])
    o2 = so.attention_rows(q[-1:], k[:, perm], v[:, perm], pos[-1:])
    np.testing.assert_allclose(o2[0], o[-1], rtol=1e-12)
    # grouped-query attention equals multi-head attention with repeated kv heads
    o3 = so.attention_rows(q, np.repeat(k, 2, axis=0), np.repeat(v, 2, axis=0), pos)
    np.testing.assert_allclose(o3, o, rtol=1e-14)
    # a key beyond a row's position has no influence on it
    k4, v4 = k.copy(), v.copy()
    k4[:, 4:], v4[:, 4:] = 99.0, -99.0
    np.testing.assert_allclose(so.attention_rows(q, k4, v4, pos)[:4], o[:4], rtol=1e-14)


def test_silu_and_greedy():
    assert so.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(so.silu(np.array([40.0, -40.0, 1.0])), [40.0, 0.0, 1 / (1 + math.exp(-1))], atol=1e-15)
    lg = np.array([[0.0, 3.0, 3.0, 1.0], [5.0, 5.0, 5.0, 5.0], [-1.0, -2.0, -0.5, -0.5]])
    assert so.greedy(lg).tolist() == [1, 0, 2]


# ----------------------------------------------------------------------------- one layer
def make_stage(s, seed=5, lo=0, hi=None, max_batch=4, max_seq=32, tensors=None):
    hi = s.n_layers_total if hi is None else hi
    st = so.OracleStage(s, lo, hi, max_batch, max_seq)
    for l in range(lo, hi):
        st.load_tensors(l, tensors[l] if tensors else synth.layer_tensors(s, seed, l))
    if st.first:
        st.load_tensors(-1, synth.embed_tensors(s, seed))
    if st.last:
        st.load_tensors(s.n_layers_total, synth.head_tensors(s, seed))
    return st


def layer_literal(s, w, x):
    """One decoder layer on one sequence from position 0: scalar loops only."""
    n, d = len(x), s.hidden
    hq, hkv, hd, F = s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn
    def norm(row, g):
        ms = sum(a * a for a in row) / d
        return [row[i] / math.sqrt(ms + s.rms_eps) * g[i] for i in range(d)]
    def matvec(W, vec):  # W is [out][in]
        return [sum(W[o][i] * vec[i] for i in range(len(vec))) for o in range(len(W))]
    def rot(vec, p):  # all heads of one row, adjacent pairs
        out = list(vec)
        for h in range(len(vec) // hd):
            for i in range(hd // 2):
                a = p * s.rope_base ** (-2.0 * i / hd)
                u0, u1 = vec[h * hd + 2 * i], vec[h * hd + 2 * i + 1]
                out[h * hd + 2 * i] = u0 * math.cos(a) - u1 * math.sin(a)
                out[h * hd + 2 * i + 1] = u0 * math.sin(a) + u1 * math.cos(a)
        return out
    Q, K, V = [], [], []
    for p in range(n):
        qkv = matvec(w["wqkv"], norm(x[p], w["attn_norm"]))
        Q.append(rot(qkv[: hq * hd], p))
        K.append(rot(qkv[hq * hd : (hq + hkv) * hd], p))
        V.append(qkv[(hq + hkv) * hd :])
    out = []
    for p in range(n):
        att = []
        for h in range(hq):
            kh = h // (hq // hkv)
            sc = [sum(Q[p][h * hd + e] * K[j][kh * hd + e] for e in range(hd)) / math.sqrt(hd) for j in range(p + 1)]
            m = max(sc)
            ex = [math.exp(a - m) for a in sc]
            att += [sum(ex[j] * V[j][kh * hd + e] for j in range(p + 1)) / sum(ex) for e in range(hd)]
        o = matvec(w["wo"], att)
        x1 = [x[p][i] + o[i] for i in range(d)]
        gu = matvec(w["wgu"], norm(x1, w["ffn_norm"]))
        hcol = [gu[f] / (1 + math.exp(-gu[f])) * gu[F + f] for f in range(F)]
        dn = matvec(w["wd"], hcol)
        out.append([x1[i] + dn[i] for i in range(d)])
    return np.array(out)


def test_layer_against_scalar_loops():
    s = TINY.with_(vocab=0, n_layers_total=1)
    t = {k: v * (1.0 if k.endswith("norm") else 20.0) for k, v in synth.layer_tensors(s, 9, 0).items()}
    st = make_stage(s, tensors={0: t})
    x = rnd(4, 5, s.hidden)
    got = st.prefill(x, [5])
    want = layer_literal(s, {k: v.astype(np.float64).tolist() for k, v in t.items()}, x.tolist())
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_layer_identity_and_closed_form_cases():
    s = synth.StageShape("f32", 1, 8, 2, 2, 4, 8, 0)  # Hkv*hd == d and F == d
    d = s.hidden
    base = {k: v.astype(np.float64) for k, v in synth.layer_tensors(s, 11, 0).items()}
    x = rnd(6, 4, d)
    # zero output and down projections: the layer is the identity on the residual stream
    t = dict(base, wo=np.zeros((d, d)), wd=np.zeros((d, d)))
    np.testing.assert_array_equal(make_stage(s, tensors={0: t}).prefill(x, [4]), x)
    # q = k = 0, v = y, Wo a non-symmetric permutation, no FFN:
    #   out = x + P * running_mean(rmsnorm(x))
    perm = np.array([3, 0, 1, 2, 7, 4, 5, 6])
    P = np.zeros((d, d)); P[np.arange(d), perm] = 1.0  # out[i] = in[perm[i]]
    wqkv = np.zeros((3 * d, d)); wqkv[2 * d :] = np.eye(d)
    t = dict(base, wqkv=wqkv, wo=P, wd=np.zeros((d, d)))
    y = so.rmsnorm(x, base["attn_norm"], s.rms_eps)
    rm = np.cumsum(y, 0) / np.arange(1, 5)[:, None]
    np.testing.assert_allclose(make_stage(s, tensors={0: t}).prefill(x, [4]), x + rm[:, perm], rtol=1e-13)
    # no attention; gate = 3*y, up = y, down a permutation:
    #   out = x + P * (silu(3y) * y): silu acts on the FIRST F rows of the stack
    wgu = np.concatenate([3.0 * np.eye(d), np.eye(d)])
    t = dict(base, wo=np.zeros((d, d)), wgu=wgu, wd=P)
    y = so.rmsnorm(x, base["ffn_norm"], s.rms_eps)
    hcol = (3 * y) / (1 + np.exp(-3 * y)) * y
    np.testing.assert_allclose(make_stage(s, tensors={0: t}).prefill(x, [4]), x + hcol[:, perm], rtol=1e-13)
    # gate weights zero: the FFN adds nothing
    t = dict(base, wo=np.zeros((d, d)), wgu=np.concatenate([np.zeros((d, d)), np.eye(d)]))
    np.testing.assert_array_equal(make_stage(s, tensors={0: t}).prefill(x, [4]), x)


# ----------------------------------------------------------------------------- the stage
def test_prefill_equals_shorter_prefill_plus_decode():
    s = TINY.with_(vocab=0)
    x = rnd(8, 9, s.hidden)
    full = make_stage(s).prefill(x, [9])
    st = make_stage(s)
    part = st.prefill(x[:6], [6])
    np.testing.assert_allclose(part, full[:6], rtol=1e-12)
    for p in range(6, 9):
        np.testing.assert_allclose(st.decode(x[p : p + 1]), full[p : p + 1], rtol=1e-11, atol=1e-13)
    assert st.seq_lens[0] == 9


def test_ragged_batch_equals_each_sequence_alone():
    s = TINY.with_(vocab=0)
    lens = [3, 7, 1, 5]
    x = rnd(9, sum(lens), s.hidden)
    st = make_stage(s)
    got = st.prefill(x, lens)
    step_in = rnd(10, 4, s.hidden)
    got_d = st.decode(step_in)
    r = 0
    for b, n in enumerate(lens):
        alone = make_stage(s)
        np.testing.assert_allclose(alone.prefill(x[r : r + n], [n]), got[r : r + n], rtol=1e-12)
        np.testing.assert_allclose(alone.decode(step_in[b : b + 1]), got_d[b : b + 1], rtol=1e-12)
        r += n


def test_split_invariance_and_last_position_logits():
    s = TINY.with_(n_layers_total=3)
    lens = [4, 6]
    tok = synth.token_ids(3, sum(lens), s.vocab)
    whole = make_stage(s)
    nt, lg = whole.prefill(tok, lens)
    nt2, lg2 = whole.decode(nt)
    for k in (1, 2):
        a, b = make_stage(s, hi=k), make_stage(s, lo=k)
        tk, lgk = b.prefill(a.prefill(tok, lens), lens)
        np.testing.assert_allclose(lgk, lg, rtol=1e-12)
        tk2, lgk2 = b.decode(a.decode(tk))
        np.testing.assert_allclose(lgk2, lg2, rtol=1e-12)
        assert tk.tolist() == nt.tolist() and tk2.tolist() == nt2.tolist()
    # logits of the last position only == row slice of a single-sequence run
    one = make_stage(s)
    _, lg_one = one.prefill(tok[:4], [4])
    np.testing.assert_allclose(lg_one[0], lg[0], rtol=1e-12)
    # embedding gather is a row lookup
    e = so.decode_values(synth.embed_tensors(s, 5)["embed"])
    mid = make_stage(s, hi=1)
    z = {k: np.zeros_like(v) if k in ("wo", "wd") else v for k, v in mid.w[0].items()}
    mid.w[0] = z
    np.testing.assert_array_equal(mid.prefill(tok, lens), e[tok])


def test_packed_equals_unpacked():
    s = TINY.with_(vocab=0)
    lay = so.layer_block_layout(s)
    x = rnd(12, 6, s.hidden)
    a, b = make_stage(s), so.OracleStage(s, 0, 2, 4, 32)
    for l in range(2):
        t = synth.layer_tensors(s, 5, l)
        buf = np.full(lay["__bytes__"][0], 0xAB, np.uint8)
        for name, (off, shp) in lay.items():
            if name != "__bytes__":
                raw = t[name].view(np.uint8).reshape(-1)
                buf[off : off + raw.size] = raw
        b.load_block(l, buf)
    np.testing.assert_array_equal(a.prefill(x, [6]), b.prefill(x, [6]))



# ----------------------------------------------------------------------------- final norm + LM head, small blocks
def identity_layers(st):
    """Zero the output and down projections: every layer leaves the residual stream alone."""
    for l in range(st.lo, st.hi):
        st.w[l] = {k: np.zeros_like(v) if k in ("wo", "wd") else v for k, v in st.w[l].items()}
    return st


def test_head_leg_against_scalar_loops_on_a_ragged_batch():
    """With identity layers the stage is embedding -> final norm -> LM head at the LAST row of
    every sequence; each logit is recomputed with plain Python loops from the raw tensors."""
    s = TINY
    st = identity_layers(make_stage(s))
    lens = [3, 1, 4]
    tok = synth.token_ids(21, sum(lens), s.vocab)
    nt, lg = st.prefill(tok, lens)
    E = so.decode_values(synth.embed_tensors(s, 5)["embed"])
    head = synth.head_tensors(s, 5)
    g, W = so.decode_values(head["final_norm"]), so.decode_values(head["lm_head"])
    assert lg.shape == (3, s.vocab)
    for b, last in enumerate([2, 3, 7]):  # rows of the packed batch that end a sequence
        x = [float(E[int(tok[last]), i]) for i in range(s.hidden)]
        ms = sum(v * v for v in x) / s.hidden
        y = [x[i] / math.sqrt(ms + s.rms_eps) * float(g[i]) for i in range(s.hidden)]
        for v in range(s.vocab):
            want = sum(y[i] * float(W[v, i]) for i in range(s.hidden))
            assert abs(lg[b, v] - want) <= 1e-12 * max(1.0, abs(want)), (b, v)
        assert int(nt[b]) == max(range(s.vocab), key=lambda v: (lg[b, v], -v))
    # a decode step takes the one new row of every sequence
    nt2, lg2 = st.decode(nt)
    for b in range(3):
        x = E[int(nt[b])]
        y = x / math.sqrt(float(np.mean(x * x)) + s.rms_eps) * g
        np.testing.assert_allclose(lg2[b], [float(np.dot(y, W[v])) for v in range(s.vocab)], rtol=1e-12, atol=1e-15)


def test_head_leg_closed_form_gain_and_orientation():
    """x = (3, 4, 0, ...) over d = 16, eps = 0: rms = 1.25, so the normalised row is (2.4, 3.2, 0, ...)
    times the gain.  The head is a shift, logits[v] = y[(v + 1) mod 16]: its transpose would
    shift the other way, a missing gain would leave 2.4 / 3.2 and move the argmax."""
    s = TINY.with_(vocab=16, rms_eps=0.0)
    gain = np.full(16, 1.0)
    gain[0], gain[1] = 1.5, 0.25
    shift = np.zeros((16, 16))
    for v in range(16):
        shift[v, (v + 1) % 16] = 1.0
    x = np.zeros((1, 16))
    x[0, 0], x[0, 1] = 3.0, 4.0
    lg = so.head_logits(x, gain, shift, 0.0)
    want = np.zeros(16)
    want[15], want[0] = 2.4 * 1.5, 3.2 * 0.25  # y0 lands on v = 15, y1 on v = 0
    np.testing.assert_allclose(lg[0], want, rtol=1e-15, atol=1e-15)
    # the same through the stage: token 7's embedding row is x, layers are identity
    st = identity_layers(make_stage(s))
    emb = rnd(8, 16, 16)
    emb[7] = x[0]
    st.w[-1] = {"embed": emb}
    st.w[s.n_layers_total] = {"final_norm": gain, "lm_head": shift}
    nt, lg = st.prefill(np.array([2, 7], np.int32), [2])
    np.testing.assert_allclose(lg[0], want, rtol=1e-15, atol=1e-15)
    assert nt.tolist() == [15]
    # eps sits inside the root here too: x = (3, 4, 0...) with eps = 9/16 gives rms = sqrt(25/16 + 9/16)
    lg_eps = so.head_logits(x, np.ones(16), np.eye(16), 9.0 / 16.0)
    np.testing.assert_allclose(lg_eps[0, :2], [3.0 / math.sqrt(34.0 / 16.0), 4.0 / math.sqrt(34.0 / 16.0)], rtol=1e-15)


def test_embed_and_head_block_layouts_hand_computed():
    # tiny fp32 benchmark config: V = 512, d = 256, 4-byte elements
    tiny = synth.CONFIGS["tiny_f32"]
    lay = so.embed_block_layout(tiny)
    assert lay["embed"] == (0, (512, 256)) and lay["__bytes__"][0] == 524288
    lay = so.head_block_layout(tiny)
    assert lay["final_norm"] == (0, (256,))
    assert lay["lm_head"] == (1024, (512, 256))
    assert lay["__bytes__"][0] == 1024 + 524288
    # bf16, d = 20, V = 50: the 40-byte gain is padded to 256; 50*20*2 = 2000 bytes pad to 2048
    odd = synth.StageShape("bf16", 1, 20, 2, 1, 4, 10, 50)
    lay = so.head_block_layout(odd)
    assert lay["final_norm"] == (0, (20,)) and lay["lm_head"] == (256, (50, 20))
    assert lay["__bytes__"][0] == 256 + 2048
    assert so.embed_block_layout(odd)["__bytes__"][0] == 2048
    # Llama-13B-shaped head: 5120 gains (10240 B, already aligned) + 32000 x 5120 bf16
    big = so.head_block_layout(synth.CONFIGS["llama13b"])
    assert big["lm_head"][0] == 10240 and big["__bytes__"][0] == 10240 + 32000 * 5120 * 2


def test_embed_and_head_blocks_load_from_packed_bytes():
    """load_block(-1) and load_block(L) on buffers assembled at hand-computed offsets (padding
    filled with junk) give the stage the same tensors as handing them over unpacked."""
    s = synth.StageShape("bf16", 1, 20, 2, 1, 4, 10, 50)
    e, h = synth.embed_tensors(s, 9), synth.head_tensors(s, 9)
    ebuf = np.full(2048, 0xAB, np.uint8)
    ebuf[:2000] = e["embed"].view(np.uint8).reshape(-1)
    hbuf = np.full(256 + 2048, 0xCD, np.uint8)
    hbuf[:40] = h["final_norm"].view(np.uint8).reshape(-1)
    hbuf[256:2256] = h["lm_head"].view(np.uint8).reshape(-1)
    a, b = so.OracleStage(s, 0, 1, 2, 8), so.OracleStage(s, 0, 1, 2, 8)
    for st in (a, b):
        st.load_tensors(0, synth.layer_tensors(s, 9, 0))
    a.load_block(-1, ebuf)
    a.load_block(1, hbuf)
    b.load_tensors(-1, e)
    b.load_tensors(1, h)
    np.testing.assert_array_equal(a.w[-1]["embed"], so.decode_values(e["embed"]))
    np.testing.assert_array_equal(a.w[1]["final_norm"], so.decode_values(h["final_norm"]))
    np.testing.assert_array_equal(a.w[1]["lm_head"], so.decode_values(h["lm_head"]))
    tok = synth.token_ids(3, 5, s.vocab)
    (ta, la), (tb, lb) = a.prefill(tok, [2, 3]), b.prefill(tok, [2, 3])
    np.testing.assert_array_equal(la, lb)
    assert ta.tolist() == tb.tolist()
    with pytest.raises(AssertionError):  # a block of the wrong size is refused
        a.load_block(1, hbuf[:-256])


def test_diagnostic_bf16_mode_is_off_by_default_and_rounds_to_nearest_even():
    f = np.array([1.0, 1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8, 1.0 + 2.0**-8 + 2.0**-20, -0.3, 3.14159])
    got = so.round_bf16(f)
    assert got[:4].tolist() == [1.0, 1.0, 1.0 + 2.0**-6, 1.0 + 2.0**-7]  # ties go to the even pattern
    assert got[4] == so.decode_values(synth.bf16_bits_from_f32(np.float32([-0.3])))[0]
    assert got[5] == 3.140625
    s = TINY.with_(vocab=0)
    x = rnd(3, 9, s.hidden)
    plain, again, rounded = make_stage(s), make_stage(s), make_stage(s)
    rounded._r, rounded._rw, rounded.round_output = so.round_bf16, so.round_bf16, True
    a, b, c = plain.prefill(x, [4, 5]), again.prefill(x, [4, 5]), rounded.prefill(x, [4, 5])
    np.testing.assert_array_equal(a, b)
    err = np.linalg.norm(c - a) / np.linalg.norm(a)
    assert 1e-4 < err < 1e-2, err  # the mode perturbs at the 16-bit level, and only when asked
    on = so.OracleStage(s, 0, 2, 4, 32, bf16_handoffs=True)
    assert on._rw is so.round_bf16 and on.round_output and so.OracleStage(s, 0, 2, 4, 32)._rw is None


# ----------------------------------------------------------------------------- planted mistakes
def _run_pins():
    for fn in (
        test_rmsnorm_closed_forms,
        test_rope_explicit_angles_and_pairing,
        test_rope_invariants,
        test_attention_brute_force_tiny,
        test_attention_special_cases,
        test_silu_and_greedy,
        test_layer_against_scalar_loops,
        test_layer_identity_and_closed_form_cases,
        test_prefill_equals_shorter_prefill_plus_decode,
        test_split_invariance_and_last_position_logits,
        test_head_leg_against_scalar_loops_on_a_ragged_batch,
        test_head_leg_closed_form_gain_and_orientation,
        test_embed_and_head_block_layouts_hand_computed,
        test_embed_and_head_blocks_load_from_packed_bytes,
    ):
        fn()


def test_planted_mistakes_are_caught(monkeypatch):
    def rope_half_split(u, pos, base):
        hd = u.shape[-1]
        th = np.power(float(base), -2.0 * np.arange(hd // 2) / hd)
        ang = np.asarray(pos, float)[:, None] * th
        c, sn = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        a, b = u[..., : hd // 2], u[..., hd // 2 :]
        return np.concatenate([a * c - b * sn, a * sn + b * c], -1)

    def rope_wrong_sign(u, pos, base):
        return so_rope(u, -np.asarray(pos), base)

    def rmsnorm_eps_outside(x, g, eps):
        return x / (np.sqrt(np.mean(x * x, -1, keepdims=True)) + eps) * g

    def attn_no_scale(q, k, v, pos):
        return so_attn(q * math.sqrt(q.shape[-1]), k, v, pos)

    def attn_strict_causal(q, k, v, pos):
        return so_attn(q, k, v, np.maximum(np.asarray(pos) - 1, 0))

    def attn_wrong_group(q, k, v, pos):
        return so_attn(q, k[::-1], v[::-1], pos)

    def silu_as_sigmoid(z):
        return 1.0 / (1.0 + np.exp(-z))

    def greedy_last(lg):
        return (lg.shape[-1] - 1 - np.argmax(lg[..., ::-1], -1)).astype(np.int32)

    def head_without_norm(x, g, w, eps):
        return x @ w.T

    def head_without_gain(x, g, w, eps):
        return so_rms(x, np.ones_like(g), eps) @ w.T

    def head_transposed(x, g, w, eps):
        return so_rms(x, g, eps) @ (w if w.shape[0] == w.shape[1] else w.T)

    def head_eps_outside(x, g, w, eps):
        return x / (np.sqrt(np.mean(x * x, -1, keepdims=True)) + eps) * g @ w.T

    def head_layout_unpadded(s):
        isz = 4 if s.dtype == "f32" else 2
        return {"final_norm": (0, (s.hidden,)), "lm_head": (s.hidden * isz, (s.vocab, s.hidden)),
                "__bytes__": (so_round(s.hidden * isz + s.vocab * s.hidden * isz, 256), ())}

    def head_layout_swapped(s):
        isz = 4 if s.dtype == "f32" else 2
        nh = so_round(s.vocab * s.hidden * isz, 256)
        return {"lm_head": (0, (s.vocab, s.hidden)), "final_norm": (nh, (s.hidden,)),
                "__bytes__": (nh + so_round(s.hidden * isz, 256), ())}

    so_rope, so_attn, so_rms, so_round = so.rope, so.attention_rows, so.rmsnorm, so._round_up
    plants = [
        ("head_logits", head_without_norm), ("head_logits", head_without_gain),
        ("head_logits", head_transposed), ("head_logits", head_eps_outside),
        ("head_block_layout", head_layout_unpadded), ("head_block_layout", head_layout_swapped),
        ("rope", rope_half_split), ("rope", rope_wrong_sign), ("rmsnorm", rmsnorm_eps_outside),
        ("attention_rows", attn_no_scale), ("attention_rows", attn_strict_causal),
        ("attention_rows", attn_wrong_group), ("silu", silu_as_sigmoid), ("greedy", greedy_last),
    ]
    _run_pins()  # green before planting anything
    for name, bad in plants:
        with monkeypatch.context() as m:
            m.setattr(so, name, bad)
            with pytest.raises(AssertionError):
                _run_pins()


def test_tiny_fp32_golden_is_reproduced():
    """The stored oracle output for benchmark config 1 (tests/golden/, written by the
    committed script from the oracle alone) is what the oracle computes today."""
    import importlib.util
    import os

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_tiny_fp32_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    prompt, toks, tops = mod.compute()
    rows = dict(l.split(" ", 1) for l in open(os.path.join(here, "tiny_fp32_greedy.txt")) if not l.startswith("#"))
    assert list(map(int, rows["prompt"].split())) == prompt
    assert list(map(int, rows["greedy"].split())) == toks
    np.testing.assert_allclose(list(map(float, rows["top_logit"].split())), tops, rtol=1e-9)
