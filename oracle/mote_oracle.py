"""CPU oracle for the forward pass of one MoTE layer (Mixture of Ternary Experts).

THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct numpy
implementation of what the GPU library computes.  Only the tests, the smoke check
and the benchmark's cpu_baseline leg may import it; the product path never does.
It shares no code, table or helper with the HIP kernels.

Every function cites the passage of the MoTE paper (arXiv 2506.14435) it follows.
Equation numbers count the displayed equations of Section 3 in order of appearance:
Eq.1-2 block forward, Eq.3 gate softmax, Eq.4 MoE sum, Eq.5-6 ternary expert,
Eq.7 Q_w, Eq.8 Q_a, Eq.9 alpha / beta, Eq.10 RoundClip.

Conventions
-----------
* bf16 tensors are numpy uint16 arrays holding the bit patterns.
* A weight matrix W is [out, in] and acts on a column vector (Section 3.1, the
  sentence after Eq.10: W in R^{m x n}).  The superscript T on W^T_up etc. in
  Eq.5-6 marks "ternary", it is not a transpose.
* Floating point is fp64 wherever the result is a real number.  The two
  quantisers decide integers, so their arithmetic is carried out in fp32 (the
  precision the kernels use): one IEEE divide for the scale, one IEEE multiply,
  round-half-to-even, clip.  The SwiGLU of a routed expert feeds a quantiser, so
  it too is evaluated in fp32 with a correctly rounded exp.
* Readings of points the paper leaves open (rounding mode, evaluation order,
  zero scales, precision of h) are listed next to the function that takes them.

Parity pins (tests/test_oracle_pins.py): every function below is pinned against
something other than itself -- closed forms, hand-worked exact cases, library
routines, brute force on tiny inputs, and the expert-memory figures of Table 1.
The paper prints no worked numerical example of the layer, so the readings R1-R3
(rounding mode, evaluation order, epsilon clamp) are pinned only against their
written statement here: "parity unpinned" with respect to the authors' own code.
"""
from __future__ import annotations

import numpy as np

EPS = np.float32(1e-5)          # clamp for alpha and beta (BitNet convention, cited in Section 3.1)
TILE_N = 32                      # packed format: rows per tile
TILE_K = 128                     # packed format: input channels per tile


# --------------------------------------------------------------------------- bf16
def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------- RoundClip
def round_clip(v: np.ndarray, lo: float, hi: float) -> np.ndarray:
    """Eq.10: max(lo, min(hi, round(v))).  Reading: round = half-to-even."""
    return np.maximum(lo, np.minimum(hi, np.rint(v)))


# ------------------------------------------------------------------- Q_w (Eq.7,9)
def absmean_scale(w: np.ndarray) -> np.float32:
    """Eq.9: alpha = ||W||_1 / (n m), one scale for the whole matrix.

    The sum runs in fp64 and is rounded to fp32 once; alpha is clamped to >= 1e-5
    so that an all-zero matrix is quantised to zeros instead of dividing by zero."""
    a = np.float32(np.sum(np.abs(np.asarray(w, dtype=np.float64))) / w.size)
    return max(a, EPS)


def ternarize(w: np.ndarray):
    """Eq.7: Q_w(W) = alpha * RoundClip(W / alpha, -1, 1).

    Returns (t, alpha): t int8 in {-1,0,1} with the shape of W, alpha fp32.
    W / alpha is one fp32 IEEE divide (Eq.7 taken literally)."""
    w32 = np.asarray(w, dtype=np.float32)
    alpha = absmean_scale(w32)
    t = round_clip(w32 / alpha, -1.0, 1.0).astype(np.int8)
    return t, alpha


# ------------------------------------------------------------------- Q_a (Eq.8,9)
def absmax_int8(x: np.ndarray):
    """Eq.8: Q_a(x) = (beta/127) * RoundClip(127 x / beta, -128, 127), beta = ||x||_inf
    per token (last axis).

    Returns (q, beta): q int8, beta fp32 [..., 1] (clamped to >= 1e-5).
    Reading: 127 x / beta is evaluated as x * (127 / beta) in fp32."""
    x32 = np.asarray(x, dtype=np.float32)
    beta = np.maximum(np.max(np.abs(x32), axis=-1, keepdims=True), EPS).astype(np.float32)
    s = (np.float32(127.0) / beta).astype(np.float32)
    q = round_clip(x32 * s, -128.0, 127.0).astype(np.int8)
    return q, beta


# ------------------------------------------------------- INT2 storage (Section 3.1)
def pack_int2(t: np.ndarray) -> np.ndarray:
    """Ternary matrix [N, K] (int8 in {-1,0,1}) -> N*K/16 uint32 words, 4 weights/byte.

    The paper says only that ternary weights are stored as INT2; the layout is this
    library's.  code = t + 1 in {0,1,2}.  The matrix is cut into tiles of 32 rows x
    128 input channels, tile (nt, kt) at word offset 256 * (nt * K/128 + kt).  In a
    tile, word 4*(32*g + r) + s holds the 16 codes of row 32*nt + r for input
    channels 128*kt + 32*s + 16*g + i, i = 0..15; code i sits at bit
    8*(i % 4) + 2*(i // 4)."""
    n_rows, n_cols = t.shape
    assert n_rows % TILE_N == 0 and n_cols % TILE_K == 0
    code = (t.astype(np.int64) + 1).astype(np.uint32)
    out = np.zeros(n_rows * n_cols // 16, dtype=np.uint32)
    tiles_k = n_cols // TILE_K
    n = np.arange(n_rows)[:, None]
    c = np.arange(n_cols)[None, :]
    nt, r = n // 32, n % 32
    kt, cc = c // 128, c % 128
    s, g, i = cc // 32, (cc % 32) // 16, cc % 16
    word = 256 * (nt * tiles_k + kt) + 4 * (32 * g + r) + s
    shift = (8 * (i % 4) + 2 * (i // 4)).astype(np.uint32)
    np.bitwise_or.at(out, word.ravel(), (code << shift).ravel())
    return out


def unpack_int2(words: np.ndarray, n_rows: int, n_cols: int) -> np.ndarray:
    """Inverse of pack_int2; raises on the unused code 3."""
    words = np.asarray(words, dtype=np.uint32)
    tiles_k = n_cols // TILE_K
    t = np.empty((n_rows, n_cols), dtype=np.int8)
    for n in range(n_rows):
        for c in range(n_cols):
            nt, r = divmod(n, 32)
            kt, cc = divmod(c, 128)
            s, g, i = cc // 32, (cc % 32) // 16, cc % 16
            wv = int(words[256 * (nt * tiles_k + kt) + 4 * (32 * g + r) + s])
            code = (wv >> (8 * (i % 4) + 2 * (i // 4))) & 3
            if code == 3:
                raise ValueError("invalid 2-bit code 3")
            t[n, c] = code - 1
    return t


def packed_bytes(n_rows: int, n_cols: int) -> int:
    """INT2 storage: 2 bits per weight, no per-group scales (Table 1 arithmetic)."""
    return n_rows * n_cols // 4


# ----------------------------------------------------------------- router (Eq.3)
def router(x_bf16: np.ndarray, w_router_bf16: np.ndarray, bias, k: int):
    """Eq.3 plus sparse top-k gating (Section 3.1, GShard-style; Section 4.1 top-k).

    x [T, d] bf16 bits, w_router [d, E] bf16 bits (the router projection stays BF16),
    bias fp32 [E] or None (None is the paper's layer).
    Returns logits fp64 [T,E], p fp64 [T,E] (softmax over all E), idx int32 [T,k]
    (k largest, descending, exact ties -> lower expert index) and w fp32 [T,k] =
    p[idx], NOT renormalised: Eq.4 multiplies by P(x)_i itself."""
    x = bf16_to_f32(x_bf16).astype(np.float64)
    wr = bf16_to_f32(w_router_bf16).astype(np.float64)
    logits = x @ wr
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]
    z = logits - logits.max(axis=1, keepdims=True)
    ez = np.exp(z)
    p = ez / ez.sum(axis=1, keepdims=True)
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :k].astype(np.int32)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1).astype(np.float32)
    return logits, p, idx, w


def dispatch_order(idx: np.ndarray, n_experts: int):
    """Expert-sorted slot order used by the boundary's row_of / tok_of outputs:
    slots are grouped by expert (ascending), and inside an expert ordered by the
    flat position t*k + j (ascending).  Returns counts [E], row_of [T,k], tok_of [R]."""
    n_tok, k = idx.shape
    flat = idx.reshape(-1)
    order = np.argsort(flat, kind="stable")
    row_of = np.empty(n_tok * k, dtype=np.int32)
    row_of[order] = np.arange(n_tok * k, dtype=np.int32)
    tok_of = (order // k).astype(np.int32)
    counts = np.bincount(flat, minlength=n_experts).astype(np.int32)
    return counts, row_of.reshape(n_tok, k), tok_of


# ------------------------------------------------ ternary linear (Section 3.1 end)
def ternary_matmul_int(t: np.ndarray, q: np.ndarray) -> np.ndarray:
    """Integer part of Y = Q_w(W) Q_a(x): acc[r, n] = sum_c t[n, c] * q[r, c], int32.

    Evaluated with an fp64 matmul of the integer-valued operands; every partial sum
    is an integer below 2^53, so the result is exact."""
    acc = q.astype(np.float64) @ t.astype(np.float64).T
    return acc.astype(np.int32)


def silu_mul_f32(g: np.ndarray, u: np.ndarray) -> np.ndarray:
    """u * SiLU(g) in fp32: u * (g / (1 + exp(-g))), exp correctly rounded."""
    g = g.astype(np.float32)
    u = u.astype(np.float32)
    with np.errstate(over="ignore"):
        e = np.exp(-g.astype(np.float64)).astype(np.float32)
    one = np.float32(1.0)
    return (u * (g / (one + e))).astype(np.float32)


def ternary_expert(x_rows_f32, t_gate, a_gate, t_up, a_up, t_down, a_down):
    """Eq.5-6 for a batch of token rows routed to one expert.

    h = Q_w(W_up) Q_a(x) (*) SiLU(Q_w(W_gate) Q_a(x)),  FFN^T(x) = Q_w(W_down) Q_a(h).
    Each ternary linear is the integer contraction times (alpha * beta / 127).
    Reading: h is rounded once to bf16 before its Q_a (activations between linears
    are bf16 tensors, like x).  Returns a dict of every intermediate."""
    q_x, beta_x = absmax_int8(x_rows_f32)
    acc_gate = ternary_matmul_int(t_gate, q_x)
    acc_up = ternary_matmul_int(t_up, q_x)
    sx = (beta_x / np.float32(127.0)).astype(np.float32)
    g = acc_gate.astype(np.float32) * (sx * np.float32(a_gate))
    u = acc_up.astype(np.float32) * (sx * np.float32(a_up))
    h_bits = f32_to_bf16(silu_mul_f32(g, u))
    q_h, beta_h = absmax_int8(bf16_to_f32(h_bits))
    acc_down = ternary_matmul_int(t_down, q_h)
    y = acc_down.astype(np.float32) * ((beta_h / np.float32(127.0)).astype(np.float32) * np.float32(a_down))
    return dict(q_x=q_x, beta_x=beta_x[:, 0], acc_gate=acc_gate, acc_up=acc_up, h=h_bits,
                q_h=q_h, beta_h=beta_h[:, 0], acc_down=acc_down, y=y.astype(np.float32))


# --------------------------------------------------------- shared expert (Eq.2)
def shared_expert(x_bf16, wg_bf16, wu_bf16, wd_bf16):
    """FFN(x) of Eq.2: the dense checkpoint's full-precision SwiGLU FFN, active for
    every token.  bf16 operands, fp64 accumulation; the hidden activation is a bf16
    tensor.  Returns (h_s bf16 bits [T,F], y_s fp64 [T,d])."""
    x = bf16_to_f32(x_bf16).astype(np.float64)
    wg = bf16_to_f32(wg_bf16).astype(np.float64)
    wu = bf16_to_f32(wu_bf16).astype(np.float64)
    wd = bf16_to_f32(wd_bf16).astype(np.float64)
    g = x @ wg.T
    u = x @ wu.T
    h = u * (g / (1.0 + np.exp(-g)))
    h_bits = f32_to_bf16(h.astype(np.float32))
    y = bf16_to_f32(h_bits).astype(np.float64) @ wd.T
    return h_bits, y


# ----------------------------------------------------------------- whole layer
def layer_forward(x_bf16, w_router_bf16, bias, k, shared, experts, tokens=None):
    """MoE(x) + FFN(x) of Eq.2 (no residual, no LayerNorm: those are the outer terms).

    shared  = (W_gate, W_up, W_down) bf16 bits, [F,d], [F,d], [d,F]
    experts = callable e -> (t_gate, a_gate, t_up, a_up, t_down, a_down) (ternary int8
              matrices [F,d], [F,d], [d,F] with their fp32 absmean scales), called
              only for experts that receive at least one of the evaluated tokens
    tokens  = optional 1-D array of token ids: experts and outputs are evaluated for
              these tokens only (each token's result depends on that token alone);
              the router always runs on all T tokens.
    Returns a dict; per-(token, slot) tensors are indexed [i, j] with i running over
    `tokens` (or all T) and j over the k selected experts."""
    n_tok = x_bf16.shape[0]
    logits, p, idx, w = router(x_bf16, w_router_bf16, bias, k)
    n_experts = w_router_bf16.shape[1]
    counts, row_of, tok_of = dispatch_order(idx, n_experts)
    sel = np.arange(n_tok) if tokens is None else np.asarray(tokens, dtype=np.int64)
    xs_bits = x_bf16[sel]
    xs = bf16_to_f32(xs_bits)
    d = xs.shape[1]
    idx_s = idx[sel]
    # hidden width of the routed experts (the shared expert may have another one)
    f_dim = experts(int(idx_s.flat[0]))[0].shape[0] if idx_s.size else shared[0].shape[0]
    ns = len(sel)
    out = dict(logits=logits, p=p, idx=idx, w=w, counts=counts, row_of=row_of, tok_of=tok_of,
               tokens=sel)
    q_x, beta_x = absmax_int8(xs)
    out["q_x"], out["beta_x"] = q_x, beta_x[:, 0]
    acc_gate = np.zeros((ns, k, f_dim), dtype=np.int32)
    acc_up = np.zeros((ns, k, f_dim), dtype=np.int32)
    h = np.zeros((ns, k, f_dim), dtype=np.uint16)
    q_h = np.zeros((ns, k, f_dim), dtype=np.int8)
    beta_h = np.zeros((ns, k), dtype=np.float32)
    acc_down = np.zeros((ns, k, d), dtype=np.int32)
    y = np.zeros((ns, k, d), dtype=np.float32)
    for e in np.unique(idx_s):
        ii, jj = np.nonzero(idx_s == e)
        r = ternary_expert(xs[ii], *experts(int(e)))
        acc_gate[ii, jj], acc_up[ii, jj], h[ii, jj] = r["acc_gate"], r["acc_up"], r["h"]
        q_h[ii, jj], beta_h[ii, jj] = r["q_h"], r["beta_h"]
        acc_down[ii, jj], y[ii, jj] = r["acc_down"], r["y"]
    h_s, y_s = shared_expert(xs_bits, *shared)
    # Eq.2 + Eq.4: only the k selected terms of the sum are non-zero (sparse gate).
    moe = np.einsum("tj,tjc->tc", w[sel].astype(np.float64), y.astype(np.float64))
    out_f64 = y_s + moe
    out.update(acc_gate=acc_gate, acc_up=acc_up, h=h, q_h=q_h, beta_h=beta_h, acc_down=acc_down,
               y=y, h_s=h_s, y_s=y_s.astype(np.float32), out_f32=out_f64.astype(np.float32),
               out_bf16=f32_to_bf16(out_f64.astype(np.float32)))
    return out
