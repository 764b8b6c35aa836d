"""GPU parity of the pieces around the layer of Section 3.1, each through the C ABI against the
CPU oracle: the post-training quantised shared expert (Section 4.3), the block of Eq.1-2
(normalisation prologue, residual epilogue), the load-balancing statistic (Eq.12), the 1-bit
routed-expert quantiser (Table 5) and the straight-through gradients of Section 3.2."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as W
from oracle import mote_oracle as O
from tests.mote_testlib import GpuProblem, OracleProblem, bits, error_metrics

pytestmark = pytest.mark.gpu

MAX_ABS_TOL = 2e-2          # bf16 output against the oracle's unrounded fp32 output
REL_L2_TOL = 5e-3
# The quantised shared expert sums integer-valued bf16 codes in fp32 and scales afterwards, the
# oracle sums dequantised weights in fp64: the pre-activations agree to about 1e-6 relative, so a
# rounding of h_s to bf16 (half a unit = 2^-9 relative) flips for well under one value in a hundred.
HS_FLIP_RATE = 1e-2


def _m():
    import paper_2506_14435_amd as M
    M.load_library()
    return M


def _log(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------ packing
@pytest.mark.parametrize("bits_", [8, 4])
@pytest.mark.parametrize("shape", [(32, 128), (96, 384), (64, 2048), (512, 256)])
def test_pack_rtn_bit_exact(shape, bits_):
    M = _m()
    g = torch.Generator().manual_seed(shape[0] * 7 + shape[1] + bits_)
    w = (torch.randn(*shape, generator=g) * 0.02).to(torch.bfloat16)
    w[3] = 0.0                                         # a zero row: clamped scale, zero codes
    w[5, 7] = 1.0                                      # an outlier that sets its row's scale
    packed, scales = M.mote_pack_rtn(w.cuda(), bits_)
    torch.cuda.synchronize()
    q, s = O.rtn_quantize(W.bf16_bits(w), bits_)
    assert np.array_equal(scales.cpu().numpy(), s)
    assert np.array_equal(packed.cpu().numpy(), O.pack_rtn(q, bits_))
    assert packed.numel() == M.mote_rtn_packed_bytes(*shape, bits_) == O.rtn_packed_bytes(*shape, bits_)


def test_pack_binary_bit_exact():
    M = _m()
    g = torch.Generator().manual_seed(77)
    w = torch.randn(96, 256, generator=g) * 0.02
    w[0, :5] = 0.0                                     # sign(0) = +1
    for t in (w, w.to(torch.bfloat16)):
        packed, alpha = M.mote_pack_ternary(t.cuda(), binary=True)
        torch.cuda.synchronize()
        tb, a = O.binarize(t.float().numpy())
        assert alpha.item() == a
        assert np.array_equal(packed.cpu().numpy().view(np.uint32), O.pack_int2(tb))


def test_layer_with_binary_experts():
    """1-bit routed experts (Table 5) through the unchanged forward: integer stages bit-exact."""
    M = _m()
    cfg = W.MoteConfig("binary_experts", 256, 384, 4, 2, 90, seed=41)
    gp, op = GpuProblem(cfg, binary_experts=True), OracleProblem(cfg, binary_experts=True)
    taps = M.alloc_taps(gp.layer, cfg.n_tokens, ("topk_idx", "row_of", "acc_gate", "acc_up", "acc_down", "q_h"))
    out = M.mote_layer_forward(gp.layer, gp.x, taps=taps)
    torch.cuda.synchronize()
    ref = op.forward()
    flat = taps["row_of"].cpu().numpy().reshape(-1)
    assert np.array_equal(taps["topk_idx"].cpu().numpy(), ref["idx"])
    for n in ("acc_gate", "acc_up"):
        assert np.array_equal(taps[n].cpu().numpy()[flat].reshape(cfg.n_tokens, cfg.top_k, -1), ref[n])
    max_abs, rel_l2 = error_metrics(bits(out), ref["out_f32"])
    _log(f"  binary experts: max-abs-err {max_abs:.3e} rel-L2 {rel_l2:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel_l2 <= REL_L2_TOL


# ------------------------------------------------------------------ load balancing (Eq.12)
@pytest.mark.parametrize("T,d,E,k,bias", [(64, 256, 4, 2, False), (1, 256, 4, 1, False), (300, 384, 8, 2, True),
                                           (2048, 896, 8, 2, False), (5000, 256, 16, 2, True), (333, 128, 33, 3, False),
                                           (8192, 2048, 16, 2, False)])
def test_router_balance_matches_oracle(T, d, E, k, bias):
    M = _m()
    g = torch.Generator().manual_seed(T + d + E)
    x = torch.randn(T, d, generator=g).to(torch.bfloat16)
    wr = (torch.randn(d, E, generator=g) * d ** -0.5).to(torch.bfloat16)
    b = (torch.randn(E, generator=g) * 0.5) if bias else None
    idx, p, counts, gate_p, gate_sum, loss = M.mote_router_balance(x.cuda(), wr.cuda(), k, None if b is None else b.cuda())
    torch.cuda.synchronize()
    _, p_o, idx_o, w_o = O.router(W.bf16_bits(x), W.bf16_bits(wr), None if b is None else b.numpy(), k)
    t_o, s_o, loss_o = O.load_balance(p_o, idx_o)
    assert np.array_equal(idx.cpu().numpy(), idx_o)
    assert np.allclose(p.cpu().numpy(), w_o, rtol=2e-6, atol=1e-9)
    assert np.array_equal(counts.cpu().numpy(), t_o)
    assert np.allclose(gate_p.cpu().numpy(), p_o, rtol=2e-6, atol=1e-9)
    assert np.allclose(gate_sum.cpu().numpy(), s_o, rtol=1e-6)
    assert loss.item() == pytest.approx(loss_o, rel=1e-6)
    # the same routing as the plain router entry point
    idx2, p2, counts2 = M.mote_router_topk(x.cuda(), wr.cuda(), k, None if b is None else b.cuda())
    assert torch.equal(idx, idx2) and torch.equal(p, p2) and torch.equal(counts, counts2)


# ------------------------------------------------------------------------- block (Eq.1-2)
def _norm_inputs(cfg, kind, seed):
    g = torch.Generator().manual_seed(seed)
    gamma = (1.0 + 0.1 * torch.randn(cfg.d_model, generator=g)).to(torch.bfloat16)
    beta = (0.05 * torch.randn(cfg.d_model, generator=g)).to(torch.bfloat16) if kind == "layer" else None
    return gamma, beta


BLOCK_CASES = [
    (W.C1, "rms"), (W.C1, "layer"),
    (W.C1.with_tokens(1, name="c1_T1"), "rms"),
    (W.C1.with_tokens(300, name="c1_T300"), "rms"),
    (W.MoteConfig("ragged_mid", 384, 640, 8, 2, 211, seed=11, outlier_channels=2), "layer"),
    (W.MoteConfig("decode_like", 512, 1408, 16, 2, 16, seed=13, bias_kind="subset", bias_subset=4), "rms"),
    (W.MoteConfig("wide_row", 2560, 256, 4, 2, 70, seed=51), "rms"),          # more chunks than threads per row
]


@pytest.mark.parametrize("cfg,kind", BLOCK_CASES, ids=lambda c: getattr(c, "name", str(c)))
def test_block_forward_matches_oracle(cfg, kind):
    """x^a is the workload's x scaled and shifted (an un-normalised hidden state); LN(x^a) bit-exact,
    routing and integer stages on LN(x^a) bit-exact, block output within the layer's tolerances."""
    M = _m()
    _log(f"block {cfg.name} {kind}")
    gp, op = GpuProblem(cfg), OracleProblem(cfg)
    gamma, beta = _norm_inputs(cfg, kind, cfg.seed + 5)
    x_a = (gp.x.float() * 3.0 + 0.25).to(torch.bfloat16)
    op.x = W.bf16_bits(x_a.cpu())
    eps = 1e-6 if kind == "rms" else 1e-5
    names = ("topk_idx", "row_of", "q_x", "beta_x", "acc_gate", "acc_up", "xn", "out_f32")
    taps = M.alloc_taps(gp.layer, cfg.n_tokens, names)
    out = M.mote_block_forward(gp.layer, x_a, gamma.cuda(), None if beta is None else beta.cuda(), eps=eps, taps=taps)
    torch.cuda.synchronize()
    norm = ("rms", W.bf16_bits(gamma), eps) if kind == "rms" else ("layer", W.bf16_bits(gamma), W.bf16_bits(beta), eps)
    ref = op.block_forward(norm)
    assert np.array_equal(bits(taps["xn"]), ref["xn"])
    assert np.array_equal(taps["topk_idx"].cpu().numpy(), ref["idx"])
    assert np.array_equal(taps["q_x"].cpu().numpy(), ref["q_x"])
    flat = taps["row_of"].cpu().numpy().reshape(-1)
    assert np.array_equal(taps["acc_gate"].cpu().numpy()[flat].reshape(cfg.n_tokens, cfg.top_k, -1), ref["acc_gate"])
    assert np.array_equal(bits(out), O.f32_to_bf16(taps["out_f32"].cpu().numpy()))
    max_abs, rel_l2 = error_metrics(bits(out), ref["block_f32"])
    # the residual raises |out|: the final bf16 rounding alone is half a unit in the last place of the largest value
    ulp = 2.0 ** (np.floor(np.log2(np.abs(ref["block_f32"]).max())) - 8)
    _log(f"  max-abs-err {max_abs:.3e} rel-L2 {rel_l2:.3e} max|ref| {np.abs(ref['block_f32']).max():.2f} half-ulp {ulp:.3e}")
    assert max_abs <= MAX_ABS_TOL + ulp and rel_l2 <= REL_L2_TOL
    # without the residual and the norm it is the layer: block(x) - x == layer(LN(x)) up to the one rounding
    lay = M.mote_layer_forward(gp.layer, taps["xn"])
    torch.cuda.synchronize()
    diff = (out.float() - x_a.float() - lay.float()).abs().max().item()
    assert diff <= 4 * ulp + 2e-2


def test_block_forward_rejects_bad_norms():
    import ctypes
    M = _m()
    lib = M.load_library()
    cfg = W.C1
    gp = GpuProblem(cfg)
    ws = gp.layer.workspace(cfg.n_tokens)
    out = torch.empty_like(gp.x)
    B = M.binding
    for norm in (B.MoteNormStruct(0, 256, None, 1e-6), B.MoteNormStruct(1, None, None, 1e-6),
                 B.MoteNormStruct(2, 256, None, 1e-5)):
        rc = lib.mote_block_forward(ctypes.byref(gp.layer.struct), ctypes.byref(norm), ctypes.c_void_p(gp.x.data_ptr()),
                                    cfg.n_tokens, ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(ws.data_ptr()),
                                    ws.numel(), None, None)
        assert rc == 1
    assert lib.mote_block_forward(ctypes.byref(gp.layer.struct), None, ctypes.c_void_p(gp.x.data_ptr()), cfg.n_tokens,
                                  ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(ws.data_ptr()), ws.numel(), None, None) == 1


# ------------------------------------------------------- quantised shared expert (Section 4.3)
def _check_rtn_layer(cfg, bits_, gp, op, tokens=None):
    M = _m()
    T = cfg.n_tokens
    names = ("topk_idx", "row_of", "acc_gate", "acc_down", "h_s", "y_s", "out_f32")
    taps = M.alloc_taps(gp.layer, T, names)
    out = M.mote_layer_forward(gp.layer, gp.x, taps=taps)
    torch.cuda.synchronize()
    ref = op.forward(tokens=tokens)
    sel = np.arange(T) if tokens is None else np.asarray(tokens)
    sel_t = torch.from_numpy(sel.astype(np.int64)).cuda()
    assert np.array_equal(taps["topk_idx"].cpu().numpy(), ref["idx"])
    hs = bits(taps["h_s"][sel_t])
    neq = hs != ref["h_s"]
    if neq.any():     # a flip moves the value by one bf16 step; sums that cancel to nearly zero keep the fp32
        a = O.bf16_to_f32(hs[neq]).astype(np.float64)          # accumulation error of their terms instead
        b = O.bf16_to_f32(ref["h_s"][neq]).astype(np.float64)
        h_max = np.abs(O.bf16_to_f32(ref["h_s"])).max()
        assert (np.abs(a - b) <= np.maximum(np.abs(a), np.abs(b)) * 2.0 ** -7 + 1e-5 * h_max).all()
    assert neq.mean() <= HS_FLIP_RATE, neq.mean()
    y_s = taps["y_s"][sel_t].cpu().numpy()
    assert np.allclose(y_s, ref["y_s"], rtol=0, atol=2e-3 + 2e-3 * np.abs(ref["y_s"]).max())
    max_abs, rel_l2 = error_metrics(bits(out[sel_t]), ref["out_f32"])
    _log(f"  INT{bits_} shared expert, T={T}: h_s flip rate {neq.mean():.2e}, max-abs-err {max_abs:.3e}, rel-L2 {rel_l2:.3e}")
    assert max_abs <= MAX_ABS_TOL and rel_l2 <= REL_L2_TOL
    return out


RTN_SMALL = [
    W.C1, W.C1.with_tokens(1, name="c1_T1"), W.C1.with_tokens(9, name="c1_T9"), W.C1.with_tokens(24, name="c1_T24"),
    W.C1.with_tokens(64, name="c1_T64"), W.C1.with_tokens(65, name="c1_T65"), W.C1.with_tokens(300, name="c1_T300"),
    W.MoteConfig("ragged_mid", 384, 640, 8, 2, 211, seed=11, outlier_channels=2),
    W.MoteConfig("decode_like", 512, 1408, 16, 2, 16, seed=13, bias_kind="subset", bias_subset=4),
    W.MoteConfig("shared_wider_T9", 256, 384, 4, 2, 9, seed=31, d_ff_shared=640),
    W.MoteConfig("shared_wider_T1100", 256, 512, 4, 2, 1100, seed=33, d_ff_shared=1152),
    W.MoteConfig("decode_wide", 2560, 1280, 8, 2, 12, seed=17),
]


@pytest.mark.parametrize("bits_", [8, 4])
@pytest.mark.parametrize("cfg", RTN_SMALL, ids=lambda c: c.name)
def test_layer_rtn_shared_small(cfg, bits_):
    _log(f"layer {cfg.name} with an INT{bits_} shared expert")
    gp, op = GpuProblem(cfg, shared_bits=bits_), OracleProblem(cfg, shared_bits=bits_)
    # the GPU's packed codes and scales are the oracle's
    for m in range(3):
        q, s = op.shared[2 * m], op.shared[2 * m + 1]
        assert np.array_equal(gp.shared[m].cpu().numpy(), O.pack_rtn(q, bits_))
        assert np.array_equal(gp.shared_scales[m].cpu().numpy(), s)
    out = _check_rtn_layer(cfg, bits_, gp, op)
    M = _m()
    out2 = M.mote_layer_forward(gp.layer, gp.x)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("bits_", [8, 4])
@pytest.mark.parametrize("T,n", [(1, 2), (4, 4), (16, 8), (64, 16)])
def test_layer_rtn_shared_config4_decode(T, n, bits_):
    """The decode shape (3B width) with a quantised shared expert: every token against the oracle."""
    cfg = W.decode_config(T, n)
    _log(f"layer {cfg.name} with an INT{bits_} shared expert")
    gp, op = GpuProblem(cfg, shared_bits=bits_), OracleProblem(cfg, shared_bits=bits_)
    _check_rtn_layer(cfg, bits_, gp, op)


@pytest.mark.parametrize("bits_", [8, 4])
def test_layer_rtn_shared_prefill_width_sampled(bits_):
    """3B width, 2048 tokens (the large-batch path: codes expanded to integer-valued bf16, scales in
    the GEMM epilogue): tokens of every 256-row tile of the shared GEMMs, first and last row of each."""
    cfg = dataclasses.replace(W.C3, name=f"c3_T2048_int{bits_}", n_tokens=2048)
    _log(f"layer {cfg.name}")
    gp, op = GpuProblem(cfg, shared_bits=bits_), OracleProblem(cfg, shared_bits=bits_)
    tokens = np.unique(np.concatenate([np.arange(0, 2048, 256), np.arange(255, 2048, 256), [1000, 1001]]))
    _check_rtn_layer(cfg, bits_, gp, op, tokens=tokens)


def test_rtn_layer_arguments_are_validated():
    import ctypes
    M = _m()
    lib = M.load_library()
    L = M.binding.MoteLayerStruct(256, 512, 512, 4, 2, *([ctypes.c_void_p(256)] * 1), None, *([ctypes.c_void_p(256)] * 7), 3)
    assert lib.mote_layer_workspace_bytes(ctypes.byref(L), 8) == 0                      # shared_bits must be 0, 8 or 4
    L.shared_bits = 8                                                                    # scales missing
    assert lib.mote_layer_forward(ctypes.byref(L), ctypes.c_void_p(256), 8, ctypes.c_void_p(256), ctypes.c_void_p(256),
                                  1 << 30, None, None) == 1
    assert lib.mote_pack_rtn(ctypes.c_void_p(256), 32, 128, 5, ctypes.c_void_p(256), ctypes.c_void_p(256), None) == 1
    assert lib.mote_pack_rtn(ctypes.c_void_p(256), 33, 128, 8, ctypes.c_void_p(256), ctypes.c_void_p(256), None) == 2
    assert lib.mote_rtn_packed_bytes(32, 128, 5) == 0


# -------------------------------------------------- straight-through gradients (Section 3.2)
def _ste_problem(R, N, K, E, seed, cuts=None):
    """Seeded inputs of one grouped ternary linear layer on its way back: latent weights ~ N(0, 0.02)
    packed on the GPU (the pack is bit-exact against the oracle elsewhere), activations ~ N(0, 1)
    quantised by the oracle's Q_a, gradient rows ~ N(0, 1) in bf16, ragged expert groups."""
    M = _m()
    g = torch.Generator().manual_seed(9000 + seed)
    rng = np.random.default_rng(9000 + seed)
    if cuts is None:
        cuts = np.sort(rng.integers(0, R + 1, E - 1))
    offsets = np.concatenate([[0], np.asarray(cuts, np.int64), [R]]).astype(np.int64)
    latents = [torch.randn(N, K, generator=g) * 0.02 for _ in range(E)]
    packed, alpha = [], []
    for w in latents:
        p, a = M.mote_pack_ternary(w.cuda())
        packed.append(p.view(torch.uint8).reshape(-1))
        alpha.append(a)
    x = torch.randn(R, K, generator=g).numpy()
    q, beta = O.absmax_int8(x)
    dy = torch.randn(R, N, generator=g).to(torch.bfloat16)
    experts = [O.ternarize(w.numpy()) for w in latents]
    return dict(offsets=offsets, packed=torch.cat(packed), alpha=torch.cat(alpha), q=q, beta=beta.reshape(-1), dy=dy,
                experts=experts)


def _ste_tight_bound(terms):
    """terms [n, S]: the products of S sampled outputs in contraction order.  The kernel adds them in
    that order, 16 at a time, in fp32: every rounding is at most 2^-24 of the running sum, which
    stays below the largest prefix sum plus one group of 16 products."""
    n = terms.shape[0]
    running = np.abs(np.cumsum(terms, axis=0)).max(axis=0) + 16.0 * np.abs(terms).max(axis=0)
    return (n / 16 + 4) * 2.0 ** -24 * running + 1e-30


def _ste_check(p, dx, dw, N, K, experts_checked=None, rows_per_expert=None):
    """dx and dw against the oracle.  Every element within the worst-case bound of an fp32 sum of
    exact products (a bf16 value times a ternary value or an int8 code; 2^-24 of sum |terms| per
    rounding), and a sample of outputs within the much tighter bound of the running sum, which is
    far below a single product: a dropped or mis-signed term would show."""
    offsets, dy_bits = p["offsets"], W.bf16_bits(p["dy"])
    E = len(p["experts"])
    for e in (range(E) if experts_checked is None else experts_checked):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        rng = np.random.default_rng(100 + e)
        rows = np.arange(lo, hi)
        if rows_per_expert is not None and len(rows) > rows_per_expert:
            rows = np.unique(np.concatenate([[lo, hi - 1], rng.choice(rows, rows_per_expert - 2, replace=False)]))
        t, alpha = p["experts"][e]
        # dX on the chosen rows, dW from all rows of the expert
        sub_dx, _, _ = O.ste_linear_backward(dy_bits[rows], [0, len(rows)], [(t, alpha)], p["q"][rows], p["beta"][rows])
        _, sub_dw, dys = O.ste_linear_backward(dy_bits[lo:hi], [0, hi - lo], [(t, alpha)], p["q"][lo:hi], p["beta"][lo:hi])
        got_dw = dw[e].cpu().numpy().astype(np.float64)
        if hi == lo:
            assert not got_dw.any(), f"expert {e} without rows"
            continue
        got_dx = dx[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
        g = O.bf16_to_f32(dy_bits[rows]).astype(np.float64)
        a64, t64 = float(alpha), t.astype(np.float64)
        bound_dx = a64 * (np.abs(g) @ np.abs(t64)) * ((N / 16 + 4) * 2.0 ** -24) + 1e-30
        assert (np.abs(got_dx - sub_dx) <= bound_dx).all(), (e, np.abs(got_dx - sub_dx).max())
        gs = O.bf16_to_f32(dys).astype(np.float64)
        q64 = p["q"][lo:hi].astype(np.float64)
        bound_dw = (np.abs(gs).T @ np.abs(q64)) * (((hi - lo) / 16 + 4) * 2.0 ** -24) + 1e-30
        assert (np.abs(got_dw - sub_dw[0]) <= bound_dw).all(), (e, np.abs(got_dw - sub_dw[0]).max())
        # sampled outputs against the bound of the running sum
        n_s = 96
        ri, ci = rng.integers(0, len(rows), n_s), rng.integers(0, K, n_s)
        terms = g[ri].T * t64[:, ci]                                  # [N, n_s]
        tight = a64 * _ste_tight_bound(terms) + np.abs(sub_dx[ri, ci]) * 2.0 ** -23
        assert (np.abs(got_dx[ri, ci] - sub_dx[ri, ci]) <= tight).all(), (e, "dx")
        assert np.median(tight) < 0.05 * a64 * np.median(np.abs(g)), (np.median(tight), a64)
        ni, ci = rng.integers(0, N, n_s), rng.integers(0, K, n_s)
        terms = gs[:, ni] * q64[:, ci]                                # [rows of e, n_s]
        tight = _ste_tight_bound(terms)
        assert (np.abs(got_dw[ni, ci] - sub_dw[0][ni, ci]) <= tight).all(), (e, "dw")
        if hi - lo >= 8:
            assert np.median(tight) < 0.05 * np.median(np.abs(gs)) * np.median(np.abs(q64)), np.median(tight)


@pytest.mark.parametrize("R,N,K,E,cuts", [(300, 256, 128, 3, None), (1000, 512, 384, 4, None),
                                          (77, 128, 256, 5, [0, 10, 10, 64]), (64, 128, 128, 1, None),
                                          (513, 384, 256, 2, [512]),
                                          (200, 128, 128, 3, [120, 200]),          # the last expert without rows
                                          (1018, 256, 256, 4, [256, 506, 762]),    # near-equal: every block padded to the longest
                                          # near-equal and unequal groups (dW: one launch, the experts are its K ranges)
                                          (1024, 256, 256, 4, [250, 510, 770]),
                                          (2100, 128, 384, 8, [300, 600, 900, 900, 1200, 1500, 1800])])
def test_ste_linear_backward_matches_oracle(R, N, K, E, cuts):
    M = _m()
    _log(f"ste backward R={R} N={N} K={K} E={E}")
    p = _ste_problem(R, N, K, E, seed=R + N + K, cuts=cuts)
    dx, dw = M.mote_ste_linear_backward(p["dy"].cuda(), p["offsets"], p["packed"].cuda(), p["alpha"].cuda(), 1,
                                        torch.from_numpy(p["q"]).cuda(), torch.from_numpy(p["beta"]).cuda(), N, K)
    torch.cuda.synchronize()
    _ste_check(p, dx, dw, N, K)


def test_ste_linear_backward_3b_gate_matrix_sampled():
    """The gate matrices of configuration 3's width (N = 11008, K = 2048) with eight experts and
    4096 dispatch rows: two experts through the oracle, every row tile boundary of theirs in dX."""
    M = _m()
    R, N, K, E = 4096, 11008, 2048, 8
    _log(f"ste backward R={R} N={N} K={K} E={E}")
    p = _ste_problem(R, N, K, E, seed=77)
    dx, dw = M.mote_ste_linear_backward(p["dy"].cuda(), p["offsets"], p["packed"].cuda(), p["alpha"].cuda(), 1,
                                        torch.from_numpy(p["q"]).cuda(), torch.from_numpy(p["beta"]).cuda(), N, K)
    torch.cuda.synchronize()
    sizes = np.diff(p["offsets"])
    chosen = [int(np.argmax(sizes)), int(np.argsort(sizes)[len(sizes) // 2])]
    _ste_check(p, dx, dw, N, K, experts_checked=chosen, rows_per_expert=24)


@pytest.mark.parametrize("R,N,K,E,cuts,what", [
    # 32 row tiles of 256 x 8 channel tiles = one round of workgroups: one K plane
    (7816, 1024, 2048, 4, [1000, 2030, 5030], "one plane"),
    # 34 row tiles x 8 channel tiles = a full round and a nearly empty one: two K planes, added afterwards
    (8192, 2048, 2048, 8, [1000, 2100, 3100, 4200, 5200, 6150, 7170], "two planes")])
def test_ste_linear_backward_grouped_dx_on_256_row_tiles(R, N, K, E, cuts, what):
    """dX of all experts in one grouped GEMM on 256 x 256 tiles: groups that end inside a tile, tiles
    that read the next group's rows, the last tile clamped at R."""
    M = _m()
    _log(f"ste backward, grouped dX on 256-row tiles ({what}) R={R} N={N} K={K} E={E}")
    p = _ste_problem(R, N, K, E, seed=R + N + E, cuts=cuts)
    dx, dw = M.mote_ste_linear_backward(p["dy"].cuda(), p["offsets"], p["packed"].cuda(), p["alpha"].cuda(), 1,
                                        torch.from_numpy(p["q"]).cuda(), torch.from_numpy(p["beta"]).cuda(), N, K)
    torch.cuda.synchronize()
    assert torch.isfinite(dx).all()
    _ste_check(p, dx, dw, N, K, experts_checked=[0, 1, E - 1], rows_per_expert=40)


def test_ste_linear_backward_dx_in_batches_of_experts():
    """With the limit on expanded weights per grouped dX launch lowered to 1 MiB the six experts go
    through in batches of two: one batch with an expert without rows, one without any row."""
    M = _m()
    R, N, K, E = 900, 512, 768, 6
    _log(f"ste backward in batches of experts R={R} N={N} K={K} E={E}")
    p = _ste_problem(R, N, K, E, seed=4242, cuts=[0, 400, 400, 400, 700])
    M.mote_tuning_set("ste_batch_mib", 1)
    try:
        dx, dw = M.mote_ste_linear_backward(p["dy"].cuda(), p["offsets"], p["packed"].cuda(), p["alpha"].cuda(), 1,
                                            torch.from_numpy(p["q"]).cuda(), torch.from_numpy(p["beta"]).cuda(), N, K)
        torch.cuda.synchronize()
    finally:
        M.mote_tuning_set("ste_batch_mib", 4095)
    _ste_check(p, dx, dw, N, K)


def test_ste_linear_backward_arguments_are_validated():
    M = _m()
    lib = M.load_library()
    import ctypes
    offs = (ctypes.c_int32 * 3)(0, 5, 9)
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    ptr = ctypes.c_void_p(buf.data_ptr())
    call = lambda o, R, N, K, E, ws_bytes: lib.mote_ste_linear_backward(ptr, o, ptr, ptr, 1, ptr, ptr, R, N, K, E, ptr, ptr, ptr,
                                                                       ctypes.c_size_t(ws_bytes), None)
    assert call(offs, 9, 100, 128, 2, 1 << 20) == 2          # N not a multiple of 128
    assert call(offs, 10, 128, 128, 2, 1 << 20) == 1         # offsets do not end at R
    assert call((ctypes.c_int32 * 3)(0, 9, 5), 5, 128, 128, 2, 1 << 20) == 1   # not ascending
    assert call(offs, 9, 128, 128, 2, 16) == 3               # workspace too small
    assert lib.mote_ste_backward_workspace_bytes(9, 128, 128, 2) > 0
    assert lib.mote_ste_backward_workspace_bytes(9, 100, 128, 2) == 0
