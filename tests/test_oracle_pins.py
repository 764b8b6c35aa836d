"""Pins for the CPU oracle: every oracle function is checked against something other
than itself -- hand-worked exact cases, closed forms, invariants, library routines,
brute force written here directly from the paper's equations (Section 3.1, Eq.2-10),
and the expert-memory figures the paper prints (Table 1, Table 3)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import mote_oracle as O

RNG = np.random.default_rng(1234)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


# ------------------------------------------------------------------------ bf16
def test_bf16_roundtrip_matches_torch():
    x = torch.randn(100_000, dtype=torch.float32) * 37.0
    x[:8] = torch.tensor([1.00390625, 1.01171875, -1.00390625, 0.0, -0.0, 3.0e38, 1e-40, 65280.0])
    want = _bits(x.to(torch.bfloat16))
    got = O.f32_to_bf16(x.numpy())
    assert np.array_equal(got, want)
    assert np.array_equal(O.bf16_to_f32(want), x.to(torch.bfloat16).to(torch.float32).numpy())


def test_bf16_ties_go_to_even():
    # 1 + 2^-8 is exactly half way between bf16 1.0 (even mantissa) and 1 + 2^-7
    assert O.f32_to_bf16(np.array([1.00390625], np.float32))[0] == 0x3F80
    # 1 + 3*2^-8 is half way between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert O.f32_to_bf16(np.array([1.01171875], np.float32))[0] == 0x3F82


# ------------------------------------------------------------------- RoundClip
def test_round_clip_half_to_even_and_clip():
    v = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 63.5, 126.5, 127.5, -128.5, 1e9, -1e9], np.float32)
    got = O.round_clip(v, -128, 127)
    assert got.tolist() == [0, 2, 2, -0.0, -2, -2, 64, 126, 127, -128, 127, -128]


# ------------------------------------------------------------------------- Q_w
def test_ternarize_hand_case_both_tie_directions():
    # alpha = (0.75+0.75+0.25+0.25)/4 = 0.5; W/alpha = 1.5, -1.5, 0.5, -0.5
    # half-to-even: 2 -> clip 1, -2 -> clip -1, 0, -0.  (half-away would give 1,-1,1,-1)
    t, a = O.ternarize(np.array([[0.75, -0.75, 0.25, -0.25]], np.float32))
    assert a == np.float32(0.5)
    assert t.tolist() == [[1, -1, 0, 0]]


def test_ternarize_brute_force_and_invariants():
    w = (RNG.standard_normal((48, 40)) * 0.02).astype(np.float32)
    t, a = O.ternarize(w)
    s = 0.0
    for v in w.ravel():
        s += abs(float(v))
    assert a == np.float32(s / w.size)
    for n in range(w.shape[0]):
        for c in range(w.shape[1]):
            r = float(np.float32(w[n, c]) / np.float32(a))       # fp32 divide
            frac = abs(r) - math.floor(abs(r))
            m = math.floor(abs(r)) + (1 if frac > 0.5 else 0)
            if frac == 0.5:
                m = math.floor(abs(r)) + (math.floor(abs(r)) % 2)
            want = max(-1, min(1, int(math.copysign(m, r))))
            assert t[n, c] == want
    assert set(np.unique(t)) <= {-1, 0, 1}
    deq = a * t.astype(np.float32)
    assert set(np.unique(deq)) <= {-a, np.float32(0), a}


def test_ternarize_gaussian_closed_form():
    sigma = 0.02
    w = (RNG.standard_normal((1000, 1000)) * sigma).astype(np.float32)
    t, a = O.ternarize(w)
    assert abs(a / (sigma * math.sqrt(2 / math.pi)) - 1) < 5e-3
    # zero <=> |w| < alpha/2: P = erf(alpha / (2 sqrt2 sigma)) = erf(sqrt(2/pi) / (2 sqrt 2))
    p0 = math.erf(math.sqrt(2 / math.pi) / (2 * math.sqrt(2)))
    assert abs((t == 0).mean() - p0) < 3e-3
    assert abs((t == 1).mean() - (t == -1).mean()) < 3e-3


def test_ternarize_scale_invariance_and_zero_matrix():
    w = (RNG.standard_normal((32, 128)) * 0.02).astype(np.float32)
    t1, a1 = O.ternarize(w)
    t2, a2 = O.ternarize(w * np.float32(8.0))          # power of two: exact
    assert np.array_equal(t1, t2) and a2 == a1 * np.float32(8.0)
    t0, a0 = O.ternarize(np.zeros((32, 128), np.float32))
    assert a0 == np.float32(1e-5) and not t0.any()
    tb, ab = O.ternarize(O.bf16_to_f32(O.f32_to_bf16(w)))   # bf16 latents are accepted as fp32 values
    assert set(np.unique(tb)) <= {-1, 0, 1}


# ------------------------------------------------------------------------ pack
def test_pack_roundtrip_no_invalid_code_and_size():
    for shape in [(32, 128), (64, 256), (96, 384)]:
        t = RNG.integers(-1, 2, size=shape).astype(np.int8)
        words = O.pack_int2(t)
        assert words.dtype == np.uint32 and words.nbytes == shape[0] * shape[1] // 4
        assert words.nbytes == O.packed_bytes(*shape)
        assert np.array_equal(O.unpack_int2(words, *shape), t)
        fields = (words[:, None] >> (2 * np.arange(16, dtype=np.uint32))[None, :]) & 3
        assert (fields != 3).all()


def test_pack_hand_computed_positions():
    # all zeros -> every 2-bit code is 1 -> every byte 0b01010101
    base = O.pack_int2(np.zeros((64, 256), np.int8))
    assert (base == 0x55555555).all()
    # row 33, channel 213: nt=1, r=1, kt=1, cc=85 -> s=2, g=1 (85%32=21>=16), i=5
    # word = 256*(1*2+1) + 4*(32*1+1) + 2 = 902 ; shift = 8*(5%4) + 2*(5//4) = 10
    t = np.zeros((64, 256), np.int8)
    t[33, 213] = 1
    diff = O.pack_int2(t) ^ base
    assert np.flatnonzero(diff).tolist() == [902]
    assert diff[902] == ((2 ^ 1) << 10)
    # row 0, channel 15: word 3? no: s=0, g=0, i=15 -> word 0, shift 8*3 + 2*3 = 30
    t = np.zeros((64, 256), np.int8)
    t[0, 15] = -1
    diff = O.pack_int2(t) ^ base
    assert np.flatnonzero(diff).tolist() == [0] and diff[0] == ((0 ^ 1) << 30)


def test_pack_is_a_bijection_on_bit_fields():
    shape = (64, 256)
    base = O.pack_int2(np.zeros(shape, np.int8))
    seen = set()
    pos = [(int(n), int(c)) for n, c in zip(RNG.integers(0, 64, 300), RNG.integers(0, 256, 300))]
    pos += [(0, 0), (31, 127), (32, 128), (63, 255), (0, 16), (0, 32), (1, 0)]
    for n, c in set(pos):
        t = np.zeros(shape, np.int8)
        t[n, c] = 1
        diff = O.pack_int2(t) ^ base
        (wi,) = np.flatnonzero(diff)
        v = int(diff[wi])
        shift = (v & -v).bit_length() - 1
        assert v == 3 << shift and shift % 2 == 0
        assert (wi, shift) not in seen
        seen.add((wi, shift))
    # operand-ready property: (word >> 2j) & 0x03030303 yields codes 4j..4j+3 in bytes 0..3
    t = RNG.integers(-1, 2, size=(32, 128)).astype(np.int8)
    words = O.pack_int2(t)
    for r, g, s in [(0, 0, 0), (5, 1, 2), (31, 1, 3)]:
        wv = int(words[4 * (32 * g + r) + s])
        for j in range(4):
            quad = (wv >> (2 * j)) & 0x03030303
            for b in range(4):
                assert ((quad >> (8 * b)) & 0xFF) - 1 == t[r, 32 * s + 16 * g + 4 * j + b]


def test_packed_size_reproduces_paper_expert_memory():
    """Table 1 / Table 3: 2 bits per routed weight and no per-group scale overhead
    reproduce every printed expert-memory figure (GiB, one decimal)."""
    rows = []
    with open(os.path.join(GOLDEN, "table1_expert_memory.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    assert len(rows) == 10
    for model, layers, d, f, method, sbits, rbits, printed in rows:
        layers, d, f, sbits, rbits = int(layers), int(d), int(f), int(sbits), int(rbits)
        per_matrix_packed = O.packed_bytes(f, d)                      # same for [F,d] and [d,F]
        assert per_matrix_packed * 4 == d * f
        if rbits == 2:
            routed = 4 * 3 * per_matrix_packed
        else:
            routed = 4 * 3 * d * f * rbits // 8
        shared = 3 * d * f * sbits // 8
        gib = layers * (routed + shared) / 2 ** 30
        assert abs(gib - float(printed)) <= 0.05 + 1e-9, (model, method, gib, printed)


# ------------------------------------------------------------------------- Q_a
def test_absmax_int8_properties():
    x = (RNG.standard_normal((64, 256)) * 3).astype(np.float32)
    q, beta = O.absmax_int8(x)
    assert q.dtype == np.int8 and q.min() >= -128 and q.max() <= 127
    assert np.array_equal(beta[:, 0], np.abs(x).max(axis=1))
    deq = (beta / np.float32(127)) * q.astype(np.float32)
    assert (np.abs(x - deq) <= beta / 254 * (1 + 1e-5)).all()
    am = np.abs(x).argmax(axis=1)
    assert (np.abs(q[np.arange(64), am].astype(int)) == 127).all()
    q2, beta2 = O.absmax_int8(x * np.float32(0.25))
    assert np.array_equal(q, q2) and np.array_equal(beta2, beta * np.float32(0.25))


def test_absmax_int8_hand_cases():
    q, beta = O.absmax_int8(np.array([[2.0, 1.0, -1.0, 0.0, -2.0]], np.float32))
    # s = 63.5: 1.0 -> 63.5 -> 64 (tie to even), -1.0 -> -64
    assert beta[0, 0] == 2.0 and q.tolist() == [[127, 64, -64, 0, -127]]
    q, beta = O.absmax_int8(np.full((1, 8), -3.0, np.float32))
    assert q.tolist() == [[-127] * 8]
    q, beta = O.absmax_int8(np.zeros((1, 8), np.float32))
    assert beta[0, 0] == np.float32(1e-5) and not q.any()
    # evaluation order x * (127/beta): brute force in fp32 scalars
    x = (RNG.standard_normal(200)).astype(np.float32)
    q, beta = O.absmax_int8(x[None, :])
    s = np.float32(127.0) / np.float32(np.abs(x).max())
    for c in range(200):
        v = float(np.float32(x[c] * s))
        assert q[0, c] == max(-128, min(127, round(v)))       # python round is half-to-even


# ---------------------------------------------------------------- integer GEMM
def test_ternary_matmul_int_is_exact():
    t = RNG.integers(-1, 2, size=(24, 96)).astype(np.int8)
    q = RNG.integers(-128, 128, size=(7, 96)).astype(np.int8)
    got = O.ternary_matmul_int(t, q)
    assert got.dtype == np.int32 and got.shape == (7, 24)
    want = np.einsum("nc,rc->rn", t.astype(np.int64), q.astype(np.int64))
    assert np.array_equal(got, want)
    for r, n in [(0, 0), (3, 17), (6, 23)]:
        assert got[r, n] == sum(int(t[n, c]) * int(q[r, c]) for c in range(96))
    # worst case magnitude stays exact
    t = np.ones((2, 18944), np.int8)
    q = np.full((1, 18944), -128, np.int8)
    assert O.ternary_matmul_int(t, q).tolist() == [[-128 * 18944] * 2]


def test_ternary_linear_equals_fake_quant_form():
    """alpha*beta/127 * (integer contraction) == Q_w(W) Q_a(x) evaluated from the
    dequantised operands of Eq.7-8 (ties the integer form to the equations)."""
    w = (RNG.standard_normal((32, 128)) * 0.02).astype(np.float32)
    x = RNG.standard_normal((5, 128)).astype(np.float32)
    t, a = O.ternarize(w)
    q, beta = O.absmax_int8(x)
    lhs = O.ternary_matmul_int(t, q).astype(np.float64) * (float(a) * beta.astype(np.float64) / 127.0)
    qw = float(a) * t.astype(np.float64)
    qa = beta.astype(np.float64) / 127.0 * q.astype(np.float64)
    rhs = qa @ qw.T
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------------- router
def _rand_bf16(shape, scale=1.0):
    return _bits((torch.from_numpy(RNG.standard_normal(shape).astype(np.float32)) * scale).to(torch.bfloat16))


def test_router_softmax_topk_properties():
    x, wr = _rand_bf16((40, 64)), _rand_bf16((64, 8), 0.125)
    logits, p, idx, w = O.router(x, wr, None, 3)
    assert np.allclose(p.sum(1), 1.0, atol=1e-14)
    # brute force logits and softmax with python floats
    xf, wf = O.bf16_to_f32(x).astype(float), O.bf16_to_f32(wr).astype(float)
    for t in (0, 17, 39):
        l = [sum(xf[t, c] * wf[c, e] for c in range(64)) for e in range(8)]
        assert np.allclose(l, logits[t], rtol=1e-12, atol=1e-13)
        z = [math.exp(v - max(l)) for v in l]
        assert np.allclose([v / sum(z) for v in z], p[t], rtol=1e-12)
        order = sorted(range(8), key=lambda e: (-l[e], e))
        assert idx[t].tolist() == order[:3]
        assert np.array_equal(w[t], np.float32(p[t][order[:3]]))     # not renormalised
    assert (w.sum(1) < 1.0).all()
    # k = 1 is argmax; k = E is a permutation sorted by probability
    _, p1, idx1, _ = O.router(x, wr, None, 1)
    assert np.array_equal(idx1[:, 0], p1.argmax(1))
    _, pE, idxE, wE = O.router(x, wr, None, 8)
    assert (np.sort(idxE, 1) == np.arange(8)).all() and (np.diff(wE.astype(np.float64), axis=1) <= 0).all()
    # a constant added to every logit changes nothing
    _, p2, idx2, _ = O.router(x, wr, np.full(8, 3.0, np.float32), 3)
    assert np.array_equal(idx2, idx) and np.allclose(p2, p, rtol=1e-12)
    # a bias can force the choice
    b = np.zeros(8, np.float32); b[[6, 2]] = [60.0, 30.0]
    _, _, idx3, _ = O.router(x, wr, b, 2)
    assert (idx3 == np.array([6, 2])).all()


def test_router_exact_ties_take_the_lower_index():
    x = _rand_bf16((16, 32))
    col = _rand_bf16((32, 1), 0.2)
    wr = np.concatenate([col, col, col, col], axis=1)            # four identical experts
    _, p, idx, w = O.router(x, wr, None, 2)
    assert (idx == np.array([0, 1])).all() and np.allclose(p, 0.25)


def test_dispatch_order_brute_force():
    idx = RNG.integers(0, 5, size=(23, 2)).astype(np.int32)
    counts, row_of, tok_of = O.dispatch_order(idx, 6)
    slots = []
    for e in range(6):
        for t in range(23):
            for j in range(2):
                if idx[t, j] == e:
                    slots.append((t, j))
    assert counts.tolist() == [sum(1 for t, j in slots if idx[t, j] == e) for e in range(6)]
    for s, (t, j) in enumerate(slots):
        assert row_of[t, j] == s and tok_of[s] == t


# ---------------------------------------------------------------------- SwiGLU
def test_silu_mul_matches_definition():
    g = np.array([-100.0, -20.0, -1.0, -0.0, 0.0, 0.5, 3.0, 50.0], np.float32)
    u = np.array([2.0, -1.0, 3.0, 1.0, 1.0, -2.0, 0.25, 1.5], np.float32)
    got = O.silu_mul_f32(g, u)
    for i in range(len(g)):
        want = float(u[i]) * float(g[i]) / (1.0 + math.exp(-float(g[i])))
        assert got[i] == pytest.approx(want, rel=3e-7, abs=1e-38)
    want_t = (torch.from_numpy(u).double() * torch.nn.functional.silu(torch.from_numpy(g).double())).numpy()
    assert np.allclose(got, want_t, rtol=3e-7, atol=1e-38)


def test_shared_expert_matches_torch_fp64():
    d, f, n = 64, 96, 9
    x, wg, wu, wd = _rand_bf16((n, d)), _rand_bf16((f, d), 0.1), _rand_bf16((f, d), 0.1), _rand_bf16((d, f), 0.1)
    h_bits, y = O.shared_expert(x, wg, wu, wd)
    tx, tg, tu, td = (torch.from_numpy(O.bf16_to_f32(a)).double() for a in (x, wg, wu, wd))
    h = (tx @ tu.T) * torch.nn.functional.silu(tx @ tg.T)          # up (*) SiLU(gate), Eq.6 order
    hb = h.float().to(torch.bfloat16)
    assert np.array_equal(h_bits, _bits(hb))
    assert np.allclose(y, (hb.double() @ td.T).numpy(), rtol=1e-12, atol=1e-14)
    # gate and up are not interchangeable: swapping them must change the result
    h_sw, _ = O.shared_expert(x, wu, wg, wd)
    assert not np.array_equal(h_sw, h_bits)


# ------------------------------------------------- layer: brute force from Eq.2-10
def _brute_force_layer(x_bits, wr_bits, k, shared_bits, latents):
    """Token by token, expert by expert, scalar loops, straight from the equations.
    Evaluates EVERY expert densely and masks by the top-k afterwards."""
    f32 = np.float32
    x = O.bf16_to_f32(x_bits)
    wr = O.bf16_to_f32(wr_bits)
    n_tok, d = x.shape
    n_exp = wr.shape[1]
    sg, su, sd = (O.bf16_to_f32(a) for a in shared_bits)
    f_dim = sg.shape[0]

    def rne(v):
        return float(round(v))                                    # python: half-to-even

    def q_w(w):                                                   # Eq.7, Eq.9
        alpha = f32(sum(abs(float(v)) for v in w.ravel()) / w.size)
        t = [[max(-1.0, min(1.0, rne(float(f32(w[n, c]) / alpha)))) for c in range(w.shape[1])]
             for n in range(w.shape[0])]
        return np.array(t), alpha

    def q_a(v):                                                   # Eq.8, Eq.9
        beta = f32(max(abs(float(a)) for a in v))
        s = f32(127.0) / beta
        return np.array([max(-128.0, min(127.0, rne(float(f32(f32(a) * s))))) for a in v]), beta

    tern = [[q_w(latents[e][m]) for m in range(3)] for e in range(n_exp)]
    out = np.zeros((n_tok, d))
    for t in range(n_tok):
        logit = [sum(float(x[t, c]) * float(wr[c, e]) for c in range(d)) for e in range(n_exp)]
        m = max(logit)
        z = [math.exp(v - m) for v in logit]
        p = [v / sum(z) for v in z]                               # Eq.3
        top = sorted(range(n_exp), key=lambda e: (-logit[e], e))[:k]
        # shared expert (Eq.2, full precision)
        g = [sum(float(x[t, c]) * float(sg[n, c]) for c in range(d)) for n in range(f_dim)]
        u = [sum(float(x[t, c]) * float(su[n, c]) for c in range(d)) for n in range(f_dim)]
        h = [u[n] * g[n] / (1.0 + math.exp(-g[n])) for n in range(f_dim)]
        h = O.bf16_to_f32(O.f32_to_bf16(np.array(h, f32))).astype(float)
        acc = [sum(h[n] * float(sd[c, n]) for n in range(f_dim)) for c in range(d)]
        # routed experts (Eq.4-6)
        qx, bx = q_a(x[t])
        for e in range(n_exp):
            (tg, ag), (tu, au), (td, ad) = tern[e]
            gi = [sum(tg[n, c] * qx[c] for c in range(d)) for n in range(f_dim)]
            ui = [sum(tu[n, c] * qx[c] for c in range(d)) for n in range(f_dim)]
            sx = f32(bx / f32(127.0))
            gv = [f32(f32(gi[n]) * f32(sx * ag)) for n in range(f_dim)]
            uv = [f32(f32(ui[n]) * f32(sx * au)) for n in range(f_dim)]
            hv = [f32(uv[n] * f32(gv[n] / f32(f32(1.0) + f32(math.exp(-float(gv[n])))))) for n in range(f_dim)]
            hv = O.bf16_to_f32(O.f32_to_bf16(np.array(hv, f32)))
            qh, bh = q_a(hv)
            di = [sum(td[c, n] * qh[n] for n in range(f_dim)) for c in range(d)]
            sc = f32(f32(bh / f32(127.0)) * ad)
            ye = [float(f32(f32(di[c]) * sc)) for c in range(d)]
            if e in top:                                          # sparse gate: Eq.4 restricted to top-k
                for c in range(d):
                    acc[c] += float(f32(p[e])) * ye[c]
        out[t] = acc
    return out


def _tiny_problem(n_tok, d, f_dim, n_exp, seed):
    rng = np.random.default_rng(seed)

    def bf(shape, s):
        return _bits((torch.from_numpy(rng.standard_normal(shape).astype(np.float32)) * s).to(torch.bfloat16))

    x = bf((n_tok, d), 1.0)
    wr = bf((d, n_exp), d ** -0.5)
    shared = (bf((f_dim, d), 0.05), bf((f_dim, d), 0.05), bf((d, f_dim), 0.05))
    latents = [[(rng.standard_normal(s) * 0.02).astype(np.float32)
                for s in ((f_dim, d), (f_dim, d), (d, f_dim))] for _ in range(n_exp)]
    return x, wr, shared, latents


def _experts_fn(latents):
    def fn(e):
        r = []
        for m in range(3):
            t, a = O.ternarize(latents[e][m])
            r += [t, a]
        return tuple(r)
    return fn


@pytest.mark.parametrize("k", [1, 2, 3])
def test_layer_two_token_brute_force(k):
    x, wr, shared, latents = _tiny_problem(2, 32, 48, 3, seed=7 + k)
    want = _brute_force_layer(x, wr, k, shared, latents)
    got = O.layer_forward(x, wr, None, k, shared, _experts_fn(latents))
    assert np.allclose(got["out_f32"], want, rtol=2e-6, atol=1e-7)
    assert np.array_equal(got["out_bf16"], O.f32_to_bf16(got["out_f32"]))


def test_layer_single_expert_reduces_to_dense_ffn():
    """E = 1, k = 1: p = 1, the layer is the shared FFN plus one ternary FFN."""
    x, wr, shared, latents = _tiny_problem(6, 32, 64, 1, seed=3)
    got = O.layer_forward(x, wr, None, 1, shared, _experts_fn(latents))
    assert (got["w"] == 1.0).all() and (got["idx"] == 0).all()
    r = O.ternary_expert(O.bf16_to_f32(x), *_experts_fn(latents)(0))
    _, y_s = O.shared_expert(x, *shared)
    assert np.allclose(got["out_f32"], y_s + r["y"], rtol=1e-6, atol=1e-7)


def test_layer_k_equals_E_is_the_dense_sum_of_eq4():
    x, wr, shared, latents = _tiny_problem(5, 32, 64, 3, seed=11)
    got = O.layer_forward(x, wr, None, 3, shared, _experts_fn(latents))
    _, p, _, _ = O.router(x, wr, None, 3)
    _, y_s = O.shared_expert(x, *shared)
    dense = y_s.copy()
    for e in range(3):
        r = O.ternary_expert(O.bf16_to_f32(x), *_experts_fn(latents)(e))
        dense += np.float32(p[:, e:e + 1]).astype(np.float64) * r["y"]
    assert np.allclose(got["out_f32"], dense, rtol=1e-6, atol=1e-7)


def test_layer_permutation_duplication_subset_and_zero_experts():
    x, wr, shared, latents = _tiny_problem(12, 32, 64, 4, seed=5)
    fn = _experts_fn(latents)
    base = O.layer_forward(x, wr, None, 2, shared, fn)
    perm = RNG.permutation(12)
    pr = O.layer_forward(x[perm], wr, None, 2, shared, fn)
    assert np.array_equal(pr["out_f32"], base["out_f32"][perm])
    xd = np.concatenate([x, x[3:4]], axis=0)
    du = O.layer_forward(xd, wr, None, 2, shared, fn)
    assert np.array_equal(du["out_f32"][12], du["out_f32"][3])
    sub = O.layer_forward(x, wr, None, 2, shared, fn, tokens=[7, 2, 9])
    assert np.array_equal(sub["out_f32"], base["out_f32"][[7, 2, 9]])
    assert np.array_equal(sub["acc_down"], base["acc_down"][[7, 2, 9]])
    # all-zero routed latents: output is the shared expert alone
    zero = [[np.zeros_like(m) for m in lat] for lat in latents]
    z = O.layer_forward(x, wr, None, 2, shared, _experts_fn(zero))
    _, y_s = O.shared_expert(x, *shared)
    assert np.allclose(z["out_f32"], y_s, rtol=1e-7, atol=0)
    # per-slot tensors agree with the dispatch order
    for t in range(12):
        for j in range(2):
            assert base["tok_of"][base["row_of"][t, j]] == t


def test_config1_runs_under_a_second_and_is_sane():
    import time
    import workloads as W
    cfg = W.C1
    x, wr = W.bf16_bits(W.make_x(cfg)), W.bf16_bits(W.make_router(cfg))
    shared = tuple(W.bf16_bits(t) for t in W.make_shared(cfg))
    tern = {}
    for e in range(cfg.n_experts):
        r = []
        for m in range(3):
            t, a = O.ternarize(W.make_latent(cfg, e, m).numpy())
            r += [t, a]
        tern[e] = tuple(r)
    t0 = time.perf_counter()
    out = O.layer_forward(x, wr, None, cfg.top_k, shared, tern.__getitem__)
    assert time.perf_counter() - t0 < 1.0
    assert out["counts"].sum() == cfg.n_tokens * cfg.top_k
    assert np.abs(out["out_f32"]).max() < 4.0
    assert np.array_equal(np.sort(out["row_of"].ravel()), np.arange(128))
