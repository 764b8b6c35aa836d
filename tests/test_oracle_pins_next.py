"""Pins for the oracle functions beyond the layer of Section 3.1: the post-training quantised
shared expert (Section 4.3, Table 3), the normalisation and residual of the block (Eq.1-2), the
load-balancing statistic (Section 3.3, Eq.12) and the 1-bit routed-expert quantiser of the
ablation (Section 4.4, Table 5).  Each function is checked against something other than itself:
hand-worked exact cases, error bounds, library routines, scalar brute force written here from
the definitions, closed forms, and the expert-memory figures of Table 3."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import mote_oracle as O

RNG = np.random.default_rng(4321)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def _bf(a, scale=1.0):
    return _bits((torch.from_numpy(np.asarray(a, np.float32)) * scale).to(torch.bfloat16))


# ------------------------------------------------------------------ RTN (Section 4.3)
def test_rtn_hand_cases_with_ties():
    # Scales that are exact in fp32, so the ties are real ties: amax = 127/128 -> s = 2^-7 (INT8),
    # amax = 1.75 -> s = 0.25 (INT4).  Every input is exact in bf16.  Half-to-even: 63.5 -> 64,
    # 2.5 -> 2, -2.5 -> -2, 3.5 -> 4, 1.5 -> 2; half-away-from-zero would give 3 and -3 for the 2.5s.
    s8 = 2.0 ** -7
    w = _bf([[127 * s8, -63.5 * s8, 2.5 * s8, -2.5 * s8, 3.5 * s8, 0.25 * s8], [0.0] * 6])
    q, s = O.rtn_quantize(w, 8)
    assert s[0] == np.float32(s8)
    assert q[0].tolist() == [127, -64, 2, -2, 4, 0]
    assert q[1].tolist() == [0] * 6 and s[1] == np.float32(1e-5) / np.float32(127.0)     # zero row: clamped scale
    w4 = _bf([[1.75, 0.625, -0.625, 0.375, -0.875, 0.0625], [-1.75, 0.875, 0.125, 0.0, 1.0, -1.125]])
    q4, s4 = O.rtn_quantize(w4, 4)                         # /0.25: 7, 2.5, -2.5, 1.5, -3.5, 0.25 | -7, 3.5, 0.5, 0, 4, -4.5
    assert s4.tolist() == [0.25, 0.25]
    assert q4[0].tolist() == [7, 2, -2, 2, -4, 0]
    assert q4[1].tolist() == [-7, 4, 0, 0, 4, -4]
    # a scale that is not exact: the quotient is taken with the ROUNDED scale, in fp32
    w3 = _bf([[1.0, -0.5, 0.3125]])
    q3, s3 = O.rtn_quantize(w3, 4)
    s_f32 = np.float32(1.0) / np.float32(7.0)              # 0.14285715, above 1/7
    assert s3[0] == s_f32
    assert q3[0].tolist() == [7, round(float(np.float32(-0.5) / s_f32)), round(float(np.float32(0.3125) / s_f32))] == [7, -3, 2]


@pytest.mark.parametrize("bits", [8, 4])
def test_rtn_scalar_brute_force_bounds_and_invariants(bits):
    qmax = 127 if bits == 8 else 7
    w_f = (RNG.standard_normal((24, 96)) * 0.02).astype(np.float32)
    w_f[3] = 0.0
    w = _bf(w_f)
    wv = O.bf16_to_f32(w)
    q, s = O.rtn_quantize(w, bits)
    for n in range(w.shape[0]):
        amax = max(max(abs(float(v)) for v in wv[n]), float(np.float32(1e-5)))
        sn = np.float32(np.float32(amax) / np.float32(qmax))
        assert s[n] == sn
        for c in range(w.shape[1]):
            want = max(-qmax, min(qmax, round(float(np.float32(wv[n, c]) / sn))))     # python: half-to-even
            assert q[n, c] == want
    assert q.min() >= -qmax and q.max() <= qmax
    # the largest element of a row maps to +-qmax, the reconstruction error is at most half a step
    nz = [n for n in range(24) if n != 3]
    assert (np.abs(q[nz]).max(axis=1) == qmax).all()
    err = np.abs(wv.astype(np.float64) - s[:, None].astype(np.float64) * q)
    # (the quotient is rounded to fp32 before the rounding to an integer: up to qmax * 2^-24 of a step more)
    assert (err <= s[:, None].astype(np.float64) * (0.5 + qmax * 2.0 ** -23)).all()
    # scaling a row by a power of two scales s and leaves the codes alone
    q2, s2 = O.rtn_quantize(_bf(wv * 4.0), bits)
    assert np.array_equal(q2[nz], q[nz]) and np.array_equal(s2[nz], s[nz] * np.float32(4.0))
    # sign symmetry
    q3, _ = O.rtn_quantize(_bf(-wv), bits)
    assert np.array_equal(q3, -q)


@pytest.mark.parametrize("bits", [8, 4])
def test_rtn_pack_roundtrip_bijection_and_hand_positions(bits):
    qmax = 127 if bits == 8 else 7
    n_rows, n_cols = 5, 128
    q = RNG.integers(-qmax, qmax + 1, size=(n_rows, n_cols)).astype(np.int8)
    raw = O.pack_rtn(q, bits)
    assert raw.dtype == np.uint8 and raw.size == O.rtn_packed_bytes(n_rows, n_cols, bits) == n_rows * n_cols * bits // 8
    assert np.array_equal(O.unpack_rtn(raw, n_rows, n_cols, bits), q)
    order = O.rtn_channel_order(n_cols, bits)
    assert sorted(order.tolist()) == list(range(n_cols))           # a permutation of the channels
    # every single weight lands in exactly one byte (INT8) / nibble (INT4), at the documented place
    for (n, c) in [(0, 0), (0, 9), (1, 17), (2, 40), (3, 63), (4, 127), (2, 72)]:
        one = np.zeros((n_rows, n_cols), np.int8)
        one[n, c] = -3
        r = O.pack_rtn(one, bits)
        nzb = np.nonzero(r)[0]
        assert len(nzb) == 1
        if bits == 8:
            grp, cc = divmod(c, 32)
            a, g, i = cc // 16, (cc % 16) // 8, cc % 8              # channel 16a + 8g + i of its group
            assert nzb[0] == n * n_cols + 32 * grp + 16 * g + 8 * a + i
            assert r[nzb[0]] == 0xFD
        else:
            grp, cc = divmod(c, 64)
            s4, g, i = cc // 16, (cc % 16) // 8, cc % 8             # channel 16s + 8g + i of its group
            pos = 64 * grp + 32 * g + 8 * s4 + i
            assert nzb[0] == (n * n_cols + pos) // 2
            assert r[nzb[0]] == (0xD << (4 * (pos % 2)))
    if bits == 4:       # the MFMA operand view: storage positions 8m .. 8m+7 of a row are one k-group
        assert order[:8].tolist() == list(range(8)) and order[8:16].tolist() == list(range(16, 24))
        assert order[32:40].tolist() == list(range(8, 16))
    else:
        assert order[:16].tolist() == list(range(8)) + list(range(16, 24))
        assert order[16:32].tolist() == list(range(8, 16)) + list(range(24, 32))


def test_rtn_sizes_reproduce_table3_expert_memory():
    """Table 3: INT8 / INT4 shared expert + ternary routed experts; the row scales (4 bytes per
    output channel) disappear in the printed rounding."""
    rows = []
    with open(os.path.join(GOLDEN, "table1_expert_memory.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    seen = 0
    for model, layers, d, f, method, sbits, rbits, printed in rows:
        layers, d, f, sbits, rbits = int(layers), int(d), int(f), int(sbits), int(rbits)
        if method != "mote" or sbits not in (8, 4):
            continue
        seen += 1
        shared = 2 * O.rtn_packed_bytes(f, d, sbits) + O.rtn_packed_bytes(d, f, sbits) + 4 * (2 * f + d)
        routed = 4 * 3 * O.packed_bytes(f, d)
        gib = layers * (shared + routed) / 2 ** 30
        assert abs(gib - float(printed)) <= 0.05 + 1e-9, (model, sbits, gib, printed)
    assert seen == 4


@pytest.mark.parametrize("bits", [8, 4])
def test_shared_expert_rtn_matches_torch_fp64_and_bounds(bits):
    d, f, n = 64, 96, 7
    x = _bf(RNG.standard_normal((n, d)))
    ws = [_bf(RNG.standard_normal(s) * 0.1) for s in ((f, d), (f, d), (d, f))]
    qs = [O.rtn_quantize(w, bits) for w in ws]
    h_bits, y = O.shared_expert_rtn(x, *qs[0], *qs[1], *qs[2])
    tx = torch.from_numpy(O.bf16_to_f32(x)).double()
    deq = [torch.from_numpy(q.astype(np.float64)) * torch.from_numpy(s.astype(np.float64))[:, None] for q, s in qs]
    g = torch.nn.functional.linear(tx, deq[0])
    u = torch.nn.functional.linear(tx, deq[1])
    hb = (u * torch.nn.functional.silu(g)).float().to(torch.bfloat16)
    assert np.array_equal(h_bits, _bits(hb))
    assert np.allclose(y, torch.nn.functional.linear(hb.double(), deq[2]).numpy(), rtol=1e-12, atol=1e-14)
    # against the unquantised expert: each pre-activation moves by at most sum_c |x_c| * s_n / 2
    xa = np.abs(O.bf16_to_f32(x).astype(np.float64)).sum(axis=1)
    g_full = O.bf16_to_f32(x).astype(np.float64) @ O.bf16_to_f32(ws[0]).astype(np.float64).T
    assert (np.abs(g.numpy() - g_full) <= 0.5 * xa[:, None] * qs[0][1][None, :].astype(np.float64) * (1 + 1e-9)).all()
    # INT8 stays close to the bf16 expert, INT4 is coarser but the same function
    _, y_full = O.shared_expert(x, *ws)
    rel = np.linalg.norm(y - y_full) / np.linalg.norm(y_full)
    assert rel < (0.02 if bits == 8 else 0.3) and rel > 0
    # routed through layer_forward the quantised shared expert replaces the bf16 one and nothing else
    rng = np.random.default_rng(5)
    wr = _bf(rng.standard_normal((d, 3)) * d ** -0.5)
    lat = [[(rng.standard_normal(s) * 0.02).astype(np.float32) for s in ((f, d), (f, d), (d, f))] for _ in range(3)]

    def experts(e):
        r = []
        for m in range(3):
            t, a = O.ternarize(lat[e][m])
            r += [t, a]
        return tuple(r)
    a = O.layer_forward(x, wr, None, 2, tuple(ws), experts)
    b = O.layer_forward(x, wr, None, 2, (*qs[0], *qs[1], *qs[2]), experts)
    assert np.array_equal(a["acc_down"], b["acc_down"]) and np.array_equal(a["idx"], b["idx"])
    assert np.allclose(b["out_f64"] - a["out_f64"], y - y_full, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- norms and block (Eq.1-2)
def test_rms_norm_and_layer_norm_match_torch_and_invariants():
    n, d = 9, 192
    x = _bf(RNG.standard_normal((n, d)) * 3.0 + 0.5)
    gamma = _bf(1.0 + 0.1 * RNG.standard_normal(d))
    beta = _bf(0.1 * RNG.standard_normal(d))
    tx, tg, tb = (torch.from_numpy(O.bf16_to_f32(a)).double() for a in (x, gamma, beta))
    want = torch.nn.functional.rms_norm(tx, (d,), tg, eps=1e-6).float().to(torch.bfloat16)
    assert np.array_equal(O.rms_norm(x, gamma, 1e-6), _bits(want))
    want = torch.nn.functional.layer_norm(tx, (d,), tg, tb, eps=1e-5).float().to(torch.bfloat16)
    assert np.array_equal(O.layer_norm(x, gamma, beta, 1e-5), _bits(want))
    # scalar definition on one row
    xv = O.bf16_to_f32(x)[2].astype(float)
    ms = sum(v * v for v in xv) / d
    row = [xv[c] / math.sqrt(ms + 1e-6) * float(O.bf16_to_f32(gamma)[c]) for c in range(d)]
    assert np.array_equal(O.rms_norm(x, gamma, 1e-6)[2], O.f32_to_bf16(np.array(row, np.float32)))
    mu = sum(xv) / d
    var = sum((v - mu) ** 2 for v in xv) / d
    row = [(xv[c] - mu) / math.sqrt(var + 1e-5) * float(O.bf16_to_f32(gamma)[c]) + float(O.bf16_to_f32(beta)[c]) for c in range(d)]
    assert np.array_equal(O.layer_norm(x, gamma, beta, 1e-5)[2], O.f32_to_bf16(np.array(row, np.float32)))
    # invariants: unit gamma -> mean square 1 (rms) / mean 0 and variance 1 (layer), up to bf16 rounding;
    # rms_norm ignores a power-of-two rescaling of x (eps negligible), layer_norm also a shift
    one, zero = _bf(np.ones(d)), _bf(np.zeros(d))
    r = O.bf16_to_f32(O.rms_norm(x, one, 0.0)).astype(np.float64)
    assert np.allclose((r * r).mean(axis=1), 1.0, atol=5e-3)
    ln = O.bf16_to_f32(O.layer_norm(x, one, zero, 0.0)).astype(np.float64)
    assert np.allclose(ln.mean(axis=1), 0.0, atol=5e-3) and np.allclose(ln.var(axis=1), 1.0, atol=1e-2)
    assert np.array_equal(O.rms_norm(_bf(O.bf16_to_f32(x) * 8.0), gamma, 0.0), O.rms_norm(x, gamma, 0.0))
    # a zero row stays zero (eps keeps the division finite)
    z = O.rms_norm(_bf(np.zeros((1, d))), gamma, 1e-6)
    assert (O.bf16_to_f32(z) == 0).all()


def test_block_forward_is_residual_plus_layer_of_the_normalised_input():
    rng = np.random.default_rng(9)
    n, d, f, e = 6, 64, 96, 4
    x_a = _bf(rng.standard_normal((n, d)) * 2.0)
    gamma = _bf(1.0 + 0.05 * rng.standard_normal(d))
    wr = _bf(rng.standard_normal((d, e)) * d ** -0.5)
    shared = tuple(_bf(rng.standard_normal(s) * 0.05) for s in ((f, d), (f, d), (d, f)))
    lat = [[(rng.standard_normal(s) * 0.02).astype(np.float32) for s in ((f, d), (f, d), (d, f))] for _ in range(e)]

    def experts(i):
        r = []
        for m in range(3):
            t, a = O.ternarize(lat[i][m])
            r += [t, a]
        return tuple(r)
    blk = O.block_forward(x_a, ("rms", gamma, 1e-6), wr, None, 2, shared, experts)
    xn = O.rms_norm(x_a, gamma, 1e-6)
    lay = O.layer_forward(xn, wr, None, 2, shared, experts)
    assert np.array_equal(blk["xn"], xn) and np.array_equal(blk["idx"], lay["idx"])
    want = O.bf16_to_f32(x_a).astype(np.float64) + lay["out_f64"]
    assert np.allclose(blk["block_f32"], want, rtol=1e-7, atol=0)
    assert np.array_equal(blk["block_bf16"], O.f32_to_bf16(blk["block_f32"]))
    # the residual is the un-normalised input: doubling x_a leaves MoE + FFN alone (rms, eps = 0)
    b0 = O.block_forward(x_a, ("rms", gamma, 0.0), wr, None, 2, shared, experts)
    b2 = O.block_forward(_bf(O.bf16_to_f32(x_a) * 2.0), ("rms", gamma, 0.0), wr, None, 2, shared, experts)
    assert np.allclose(b2["block_f32"] - b0["block_f32"], O.bf16_to_f32(x_a), rtol=0, atol=1e-5)
    # token subset and the literal layer normalisation
    sub = O.block_forward(x_a, ("layer", gamma, _bf(np.zeros(d)), 1e-5), wr, None, 2, shared, experts, tokens=[4, 1])
    full = O.block_forward(x_a, ("layer", gamma, _bf(np.zeros(d)), 1e-5), wr, None, 2, shared, experts)
    assert np.array_equal(sub["block_f32"], full["block_f32"][[4, 1]])


# ---------------------------------------------------------------- load balancing (Eq.12)
def test_load_balance_brute_force_and_closed_forms():
    n_tok, n_exp, k = 37, 5, 2
    logits = RNG.standard_normal((n_tok, n_exp))
    p = np.exp(logits) / np.exp(logits).sum(axis=1, keepdims=True)
    idx = np.argsort(-logits, axis=1)[:, :k]
    t, s, loss = O.load_balance(p, idx)
    # Eq.12 term by term
    tt = [0] * n_exp
    for x in range(n_tok):
        for j in range(k):
            tt[int(idx[x, j])] += 1
    want = 0.0
    for i in range(n_exp):
        for x in range(n_tok):
            want += tt[i] * float(p[x, i])
    want *= n_exp / n_tok
    assert t.tolist() == tt and t.sum() == n_tok * k
    assert loss == pytest.approx(want, rel=1e-12)
    assert np.allclose(s, [sum(float(p[x, i]) for x in range(n_tok)) for i in range(n_exp)], rtol=1e-12)
    assert s.sum() == pytest.approx(n_tok, rel=1e-12)              # every row of P sums to one
    # uniform gate: sum_x P_i = |X|/E, so L = E/|X| * (|X|/E) * sum_i t_i = k |X| whatever the routing
    pu = np.full((n_tok, n_exp), 1.0 / n_exp)
    assert O.load_balance(pu, idx)[2] == pytest.approx(k * n_tok, rel=1e-12)
    # one-hot gate that agrees with top-1 routing: L = E/|X| * sum_i t_i^2, minimal (= |X|) when balanced
    n_tok = 40
    idx1 = (np.arange(n_tok) % n_exp).reshape(-1, 1)
    p1 = np.eye(n_exp)[idx1[:, 0]]
    assert O.load_balance(p1, idx1)[2] == pytest.approx(n_exp / n_tok * n_exp * (n_tok / n_exp) ** 2, rel=1e-12)
    idx_all0 = np.zeros((n_tok, 1), np.int64)
    assert O.load_balance(np.eye(n_exp)[idx_all0[:, 0]], idx_all0)[2] == pytest.approx(n_exp * n_tok, rel=1e-12)
    # the normalisation of the work the paper follows: loss / |X| equals 1 for the balanced one-hot case
    assert O.load_balance(p1, idx1)[2] / n_tok == pytest.approx(1.0, rel=1e-12)


# ------------------------------------------------------- 1-bit routed experts (Table 5)
def test_binarize_hand_case_and_invariants():
    t, a = O.binarize(np.array([[0.75, -0.25, 0.0, -0.5]], np.float32))
    assert a == np.float32(0.375) and t.tolist() == [[1, -1, 1, -1]]
    w = (RNG.standard_normal((40, 64)) * 0.02).astype(np.float32)
    t, a = O.binarize(w)
    assert set(np.unique(t).tolist()) == {-1, 1}
    assert a == np.float32(np.abs(w.astype(np.float64)).mean())
    assert np.array_equal(t, np.sign(w).astype(np.int8))            # no exact zeros in a Gaussian draw
    # alpha * sign(W) is the least-squares binary approximation: its residual is orthogonal to sign(W)
    resid = w.astype(np.float64) - float(a) * t
    assert abs((resid * t).sum()) <= 1e-6 * np.abs(w).sum()
    # the binary codes fit the INT2 container of the ternary experts (code = t + 1 in {0, 2})
    words = O.pack_int2(np.pad(t, ((0, 24), (0, 64)), constant_values=1))
    assert np.array_equal(O.unpack_int2(words, 64, 128)[:40, :64], t)
    t0, a0 = O.binarize(np.zeros((4, 4), np.float32))
    assert (t0 == 1).all() and a0 == np.float32(1e-5)


# ------------------------------------------------- straight-through gradients (Section 3.2)
def _ste_case(seed, R=11, N=12, K=10, E=3, exact_scale=False):
    rng = np.random.default_rng(seed)
    cuts = np.sort(rng.integers(0, R + 1, E - 1))
    offsets = np.concatenate([[0], cuts, [R]])
    dy = _bf(rng.standard_normal((R, N)))
    experts = [(rng.integers(-1, 2, (N, K)).astype(np.int8), np.float32(rng.uniform(0.01, 0.05))) for _ in range(E)]
    x = rng.standard_normal((R, K)).astype(np.float32)
    if exact_scale:                       # absmax 127 * 2^-5: beta / 127 = 2^-5, a power of two
        x = np.clip(x, -3.0, 3.0)
        x[:, 0] = 127.0 * 2.0 ** -5
    q, beta = O.absmax_int8(x)
    return dy, offsets, experts, q, beta.reshape(-1)


def test_ste_backward_is_the_gradient_of_the_dequantised_bilinear_form():
    """With the quantisers skipped (Section 3.2) the layer is Y = Xq Wq^T, whose gradients autograd
    (a library routine) gives: dXq = dY Wq and dWq = dY^T Xq.  The scale of each row is a power
    of two here, so folding it into the bf16 gradient row is exact and the match is to rounding."""
    dy, offsets, experts, q, beta = _ste_case(1, exact_scale=True)
    assert np.all(beta == np.float32(127.0 * 2.0 ** -5))
    dx, dw, _ = O.ste_linear_backward(dy, offsets, experts, q, beta)
    dy_t = torch.from_numpy(O.bf16_to_f32(dy).astype(np.float64))
    for e, (t, alpha) in enumerate(experts):
        lo, hi = offsets[e], offsets[e + 1]
        xq = torch.tensor(q[lo:hi].astype(np.float64) * (float(beta[0]) / 127.0), requires_grad=True)
        wq = torch.tensor(t.astype(np.float64) * float(alpha), requires_grad=True)
        y = xq @ wq.T
        y.backward(dy_t[lo:hi])
        assert np.allclose(dx[lo:hi], xq.grad.numpy(), rtol=1e-13, atol=1e-15)
        # dW is the gradient w.r.t. Q_w(W) = alpha * t itself (not w.r.t. t): no factor alpha
        assert np.allclose(dw[e], wq.grad.numpy(), rtol=1e-13, atol=1e-15)


def test_ste_backward_finite_differences_and_scalar_loops():
    """Central differences of L = sum(G * Y) in single entries of Q_a(X) and Q_w(W) (L is bilinear,
    so the difference quotient is exact up to rounding), and the two sums written as scalar loops."""
    dy, offsets, experts, q, beta = _ste_case(2, R=7, N=5, K=6, E=2, exact_scale=True)
    dx, dw, dys = O.ste_linear_backward(dy, offsets, experts, q, beta)
    g = O.bf16_to_f32(dy).astype(np.float64)
    s = beta.astype(np.float64) / 127.0

    def loss(xq, wqs):
        return sum(float((g[offsets[e]:offsets[e + 1]] * (xq[offsets[e]:offsets[e + 1]] @ wqs[e].T)).sum())
                   for e in range(len(experts)))

    xq = q.astype(np.float64) * s[:, None]
    wqs = [t.astype(np.float64) * float(a) for t, a in experts]
    h = 0.5
    for (r, c) in [(0, 0), (3, 4), (6, 5)]:
        xp, xm = xq.copy(), xq.copy()
        xp[r, c] += h
        xm[r, c] -= h
        assert math.isclose((loss(xp, wqs) - loss(xm, wqs)) / (2 * h), dx[r, c], rel_tol=1e-12, abs_tol=1e-14)
    for (e, n, c) in [(0, 0, 0), (1, 4, 5), (1, 2, 3)]:
        wp = [w.copy() for w in wqs]
        wm = [w.copy() for w in wqs]
        wp[e][n, c] += h
        wm[e][n, c] -= h
        assert math.isclose((loss(xq, wp) - loss(xq, wm)) / (2 * h), dw[e][n, c], rel_tol=1e-12, abs_tol=1e-14)
    for e, (t, alpha) in enumerate(experts):
        for r in range(offsets[e], offsets[e + 1]):
            for c in range(q.shape[1]):
                want = sum(g[r, n] * float(alpha) * int(t[n, c]) for n in range(t.shape[0]))
                assert math.isclose(dx[r, c], want, rel_tol=1e-12, abs_tol=1e-14)
        for n in range(t.shape[0]):
            for c in range(q.shape[1]):
                want = sum(g[r, n] * s[r] * int(q[r, c]) for r in range(offsets[e], offsets[e + 1]))
                assert math.isclose(dw[e][n, c], want, rel_tol=1e-12, abs_tol=1e-14)


def test_ste_backward_scale_folding_rounds_once_and_empty_experts():
    """A scale that is not a power of two: the gradient row carries it, rounded once to bf16 (half
    an ulp, at most 2^-8 relative), so dW stays within that of the unrounded sum; an expert without rows
    gets a zero dW and touches no row of dX."""
    dy, offsets, experts, q, beta = _ste_case(3, R=16, N=8, K=9, E=4)
    offsets = np.array([0, 5, 5, 12, 16])              # expert 1 has no rows
    dx, dw, dys = O.ste_linear_backward(dy, offsets, experts, q, beta)
    g = O.bf16_to_f32(dy).astype(np.float64)
    s32 = (beta / np.float32(127.0)).astype(np.float32)
    want_bits = _bits(torch.from_numpy((O.bf16_to_f32(dy) * s32[:, None]).astype(np.float32)).to(torch.bfloat16))
    assert np.array_equal(dys, want_bits)              # torch's fp32 -> bf16 conversion rounds to nearest even
    assert not dw[1].any()
    for e in (0, 2, 3):
        lo, hi = offsets[e], offsets[e + 1]
        terms = g[lo:hi, :, None] * s32.astype(np.float64)[lo:hi, None, None] * q[lo:hi, None, :].astype(np.float64)
        exact = terms.sum(axis=0)
        assert np.all(np.abs(dw[e] - exact) <= 2.0 ** -8 * np.abs(terms).sum(axis=0) + 1e-18)
        assert np.abs(dw[e] - exact).max() > 0          # the rounding is really there
    # a sign flip of one ternary weight moves exactly one column of one expert's dX rows
    t2 = experts[0][0].copy()
    t2[3, 4] = -1 if t2[3, 4] >= 0 else 1
    dx2, _, _ = O.ste_linear_backward(dy, offsets, [(t2, experts[0][1])] + experts[1:], q, beta)
    diff = np.argwhere(dx2 != dx)
    assert set(diff[:, 1]) == {4} and set(diff[:, 0]) <= set(range(0, 5))
