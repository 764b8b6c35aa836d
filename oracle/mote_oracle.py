"""CPU oracle for the forward pass of one MoTE layer (Mixture of Ternary Experts).

THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct numpy
implementation of what the GPU library computes.  Only the tests, the smoke check
and the benchmark's cpu_baseline leg may import it; the product path never does.
It shares no code, table or helper with the HIP kernels.

Every function cites the passage of the MoTE paper (arXiv 2506.14435) it follows.
Equation numbers count the displayed equations of Section 3 in order of appearance:
Eq.1-2 block forward, Eq.3 gate softmax, Eq.4 MoE sum, Eq.5-6 ternary expert,
Eq.7 Q_w, Eq.8 Q_a, Eq.9 alpha / beta, Eq.10 RoundClip, Eq.11 language-modelling loss,
Eq.12 load-balancing loss, Eq.13 total loss.

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

Parity pins (tests/test_oracle_pins.py, tests/test_oracle_pins_next.py): every function
below is pinned against something other than itself -- closed forms, hand-worked exact
cases, library routines, brute force on tiny inputs, and the expert-memory figures of
Table 1 and Table 3.
The paper prints no worked numerical example of the layer, so the readings R1-R3
(rounding mode, evaluation order, epsilon clamp) are pinned only against their
written statement here: "parity unpinned" with respect to the authors' own code.
The same holds for the readings taken beyond Section 3.1: the granularity and rounding
of the RTN shared expert (Section 4.3 names the method only), RMSNorm as the LN of
Eq.1-2, the count t_i in Eq.12, sign(0) = +1 of the 1-bit quantiser, and the operand
precision of the straight-through gradients of Section 3.2.
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


# ------------------------------------- post-training quantised shared expert (Section 4.3)
def rtn_quantize(w_bf16: np.ndarray, n_bits: int):
    """Round-to-nearest weight quantisation of a shared-expert matrix to INT8 or INT4
    (Section 4.3 and Table 3: the shared expert is quantised with RTN).

    The paper names the method only.  Reading: weight-only, symmetric, one scale per output
    channel (row of W [out, in]), the vector-wise absmax scheme of the work it cites for RTN:
        amax_n = max(max_c |W[n, c]|, 1e-5),  s_n = amax_n / qmax   (fp32 divide),
        q[n, c] = RoundClip(W[n, c] / s_n, -qmax, qmax)             (fp32 divide, Eq.10's RoundClip),
    qmax = 127 (INT8) or 7 (INT4); activations stay bf16; dequantised weight = s_n * q.
    Returns (q int8 [N, K], s fp32 [N])."""
    assert n_bits in (8, 4)
    qmax = np.float32(127.0 if n_bits == 8 else 7.0)
    w = bf16_to_f32(w_bf16)
    amax = np.maximum(np.max(np.abs(w), axis=1, keepdims=True), EPS).astype(np.float32)
    s = (amax / qmax).astype(np.float32)
    q = round_clip((w / s).astype(np.float32), -float(qmax), float(qmax)).astype(np.int8)
    return q, s[:, 0]


def rtn_packed_bytes(n_rows: int, n_cols: int, n_bits: int) -> int:
    """Bytes of the integer codes of an RTN matrix (the fp32 row scales, 4 * n_rows bytes,
    come on top and are what Table 3's rounding hides)."""
    return n_rows * n_cols * n_bits // 8


def rtn_channel_order(n_cols: int, n_bits: int) -> np.ndarray:
    """Storage order of the input channels inside a packed RTN row (this library's layout; the
    paper fixes none).  order[p] is the channel stored at position p.

    INT8: groups of 32 channels; position 16*g + 8*a + i holds channel 16*a + 8*g + i of the group
    (g, a in {0,1}, i in 0..7).  INT4: groups of 64 channels; position 32*g + 8*s + i holds channel
    16*s + 8*g + i of the group (g in {0,1}, s in 0..3, i in 0..7)."""
    grp = 32 if n_bits == 8 else 64
    assert n_cols % grp == 0
    pos = np.arange(grp)
    if n_bits == 8:
        g, a, i = pos // 16, (pos // 8) % 2, pos % 8
        ch = 16 * a + 8 * g + i
    else:
        g, s4, i = pos // 32, (pos // 8) % 4, pos % 8
        ch = 16 * s4 + 8 * g + i
    return (np.arange(0, n_cols, grp)[:, None] + ch[None, :]).reshape(-1)


def pack_rtn(q: np.ndarray, n_bits: int) -> np.ndarray:
    """RTN codes [N, K] int8 -> bytes, row-major over rows, channels in rtn_channel_order.
    INT8: one two's-complement byte per weight.  INT4: two's-complement nibbles, the code at
    storage position p of a row in byte p // 2, bits 4*(p % 2) .. 4*(p % 2) + 3."""
    n_rows, n_cols = q.shape
    qs = q[:, rtn_channel_order(n_cols, n_bits)]
    if n_bits == 8:
        return qs.astype(np.int8).view(np.uint8).reshape(-1).copy()
    nib = (qs.astype(np.int16) & 0xF).astype(np.uint8)
    return (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8).reshape(-1)


def unpack_rtn(raw: np.ndarray, n_rows: int, n_cols: int, n_bits: int) -> np.ndarray:
    """Inverse of pack_rtn (plain loops)."""
    raw = np.asarray(raw, dtype=np.uint8)
    order = rtn_channel_order(n_cols, n_bits)
    q = np.empty((n_rows, n_cols), dtype=np.int8)
    for n in range(n_rows):
        for p in range(n_cols):
            if n_bits == 8:
                v = int(raw[n * n_cols + p])
                v = v - 256 if v >= 128 else v
            else:
                b = int(raw[(n * n_cols + p) // 2])
                v = (b >> (4 * (p % 2))) & 0xF
                v = v - 16 if v >= 8 else v
            q[n, order[p]] = v
    return q


def shared_expert_rtn(x_bf16, qg, sg, qu, su, qd, sd):
    """FFN(x) of Eq.2 with the three matrices replaced by their RTN dequantisations s_n * q
    (exact in fp64); bf16 activations, fp64 accumulation, bf16 hidden activation, as in
    shared_expert.  Returns (h_s bf16 bits [T,F], y_s fp64 [T,d])."""
    x = bf16_to_f32(x_bf16).astype(np.float64)
    wg = sg.astype(np.float64)[:, None] * qg.astype(np.float64)
    wu = su.astype(np.float64)[:, None] * qu.astype(np.float64)
    wd = sd.astype(np.float64)[:, None] * qd.astype(np.float64)
    g = x @ wg.T
    u = x @ wu.T
    h = u * (g / (1.0 + np.exp(-g)))
    h_bits = f32_to_bf16(h.astype(np.float32))
    y = bf16_to_f32(h_bits).astype(np.float64) @ wd.T
    return h_bits, y


# ------------------------------------------------- normalisation of Eq.1-2 (block prologue)
def rms_norm(x_bf16, gamma_bf16, eps: float) -> np.ndarray:
    """LN(.) of Eq.1-2 for a base model whose normalisation is RMSNorm (the Qwen2.5 models the
    paper up-cycles): y = x / sqrt(mean_c x^2 + eps) * gamma, in fp64, rounded once to bf16
    (the normalised hidden state is a bf16 tensor like every activation between modules)."""
    x = bf16_to_f32(x_bf16).astype(np.float64)
    g = bf16_to_f32(gamma_bf16).astype(np.float64)
    y = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g
    return f32_to_bf16(y.astype(np.float32))


def layer_norm(x_bf16, gamma_bf16, beta_bf16, eps: float) -> np.ndarray:
    """LN(.) of Eq.1-2 taken literally as layer normalisation: (x - mean) / sqrt(var + eps) *
    gamma + beta over the channels (biased variance), fp64, rounded once to bf16."""
    x = bf16_to_f32(x_bf16).astype(np.float64)
    g = bf16_to_f32(gamma_bf16).astype(np.float64)
    b = bf16_to_f32(beta_bf16).astype(np.float64)
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps) * g + b
    return f32_to_bf16(y.astype(np.float32))


# ------------------------------------------------------- load balancing (Section 3.3, Eq.12)
def load_balance(p: np.ndarray, idx: np.ndarray):
    """Eq.12 as printed: L_balance = E / |X| * sum_i sum_x t_i * P(x)_i, with t_i the number of
    tokens routed to expert i (over all k slots) and P(x)_i the gate softmax of Eq.3.

    p [T, E] gate probabilities, idx [T, k] selected experts.
    Returns (t int64 [E], s fp64 [E] = sum_x P(x)_i, loss fp64).  The loss of the work the paper
    follows here divides by |X| once more (t_i as a fraction of the tokens): loss / T."""
    n_tok, n_exp = p.shape
    t = np.bincount(idx.reshape(-1), minlength=n_exp).astype(np.int64)
    s = p.astype(np.float64).sum(axis=0)
    loss = float(n_exp) / float(n_tok) * float(np.sum(t.astype(np.float64) * s))
    return t, s, loss


# ------------------------------------------------ 1-bit routed experts (Section 4.4, Table 5)
def binarize(w: np.ndarray):
    """The 1-bit weight quantiser of the routed-expert ablation (binary weight network of the
    work cited there): W_b = alpha * sign(W), alpha = ||W||_1 / (n m) as in Eq.9.
    Reading: sign(0) = +1 (a binary code has no zero); alpha clamped to >= 1e-5 like Q_w.
    Returns (t int8 in {-1, +1}, alpha fp32)."""
    w32 = np.asarray(w, dtype=np.float32)
    alpha = absmean_scale(w32)
    t = np.where(w32 < 0, -1, 1).astype(np.int8)
    return t, alpha


# ----------------------------------------------------------------- whole layer

def ste_linear_backward(dy_bf16, offsets, experts, q, beta):
    """Straight-through estimator of Section 3.2 for the grouped ternary linear layer of
    Section 3.1, Y_e = Q_a(X_e) Q_w(W_e)^T (rows grouped by expert e, offsets[e] .. offsets[e+1]):
    the quantisers are skipped on the way back, dL/dW = dL/dQ_w(W) and dL/dX = dL/dQ_a(X), so

        dX[r, c]   = sum_n dY[r, n] * (alpha_e * t_e[n, c])                    (gradient w.r.t. Q_a(X))
        dW_e[n, c] = sum_{r in e} dY[r, n] * ((beta_r / 127) * q[r, c])        (gradient w.r.t. Q_w(W))

    dy_bf16: bit patterns [R, N]; experts: list of (t [N, K] in {-1,0,1}, alpha fp32);
    q int8 [R, K], beta fp32 [R] or [R, 1] (the clamped absmax of Q_a).  Returns dX fp64 [R, K],
    dW fp64 [E, N, K] and the scaled gradient rows as bf16 bit patterns.
    Reading (the paper states only the two identities and that gradients stay in full
    precision): the sums run over bf16 operands with a wide accumulator, as a mixed-precision
    trainer computes them; the activation scale beta_r / 127 (one fp32 divide, as in the forward
    pass) is folded into the gradient row, dYs[r, n] = bf16(fp32(dY[r, n]) * (beta_r / 127)), one
    fp32 multiply and one rounding, because the contraction index of dW is r and a scale per r
    cannot be applied after the sum; int8 codes and ternary values are exact in bf16.  alpha_e
    multiplies the finished sum."""
    dy = bf16_to_f32(dy_bf16)
    R, N = dy.shape
    K = q.shape[1]
    scale = (np.asarray(beta, np.float32).reshape(-1) / np.float32(127.0)).astype(np.float32)
    dys_bits = f32_to_bf16((dy * scale[:, None]).astype(np.float32))
    dys = bf16_to_f32(dys_bits).astype(np.float64)
    dx = np.zeros((R, K), np.float64)
    dw = np.zeros((len(experts), N, K), np.float64)
    for e, (t, alpha) in enumerate(experts):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        dx[lo:hi] = float(np.float32(alpha)) * (dy[lo:hi].astype(np.float64) @ t.astype(np.float64))
        dw[e] = dys[lo:hi].T @ q[lo:hi].astype(np.float64)
    return dx, dw, dys_bits


def layer_forward(x_bf16, w_router_bf16, bias, k, shared, experts, tokens=None):
    """MoE(x) + FFN(x) of Eq.2 (no residual, no LayerNorm: those are the outer terms).

    shared  = (W_gate, W_up, W_down) bf16 bits, [F,d], [F,d], [d,F]; or, for a post-training
              quantised shared expert (Section 4.3), (q_gate, s_gate, q_up, s_up, q_down, s_down)
              as returned by rtn_quantize
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
    h_s, y_s = shared_expert(xs_bits, *shared) if len(shared) == 3 else shared_expert_rtn(xs_bits, *shared)
    # Eq.2 + Eq.4: only the k selected terms of the sum are non-zero (sparse gate).
    moe = np.einsum("tj,tjc->tc", w[sel].astype(np.float64), y.astype(np.float64))
    out_f64 = y_s + moe
    out.update(acc_gate=acc_gate, acc_up=acc_up, h=h, q_h=q_h, beta_h=beta_h, acc_down=acc_down,
               y=y, h_s=h_s, y_s=y_s.astype(np.float32), out_f64=out_f64, out_f32=out_f64.astype(np.float32),
               out_bf16=f32_to_bf16(out_f64.astype(np.float32)))
    return out


def block_forward(x_a_bf16, norm, w_router_bf16, bias, k, shared, experts, tokens=None):
    """The MoE half of a block, Eq.2: x_l = x^a + MoE(LN(x^a)) + FFN(LN(x^a)).

    norm = ("rms", gamma, eps) or ("layer", gamma, beta, eps); the other arguments as in
    layer_forward.  The normalised hidden state is a bf16 tensor; the residual x^a enters the
    fp64 sum unrounded and the result is rounded once to bf16.
    Returns layer_forward's dict for the normalised input plus xn (bf16 bits, all tokens) and
    block_f32 / block_bf16 for the evaluated tokens."""
    if norm[0] == "rms":
        xn = rms_norm(x_a_bf16, norm[1], norm[2])
    elif norm[0] == "layer":
        xn = layer_norm(x_a_bf16, norm[1], norm[2], norm[3])
    else:
        raise ValueError(norm[0])
    out = layer_forward(xn, w_router_bf16, bias, k, shared, experts, tokens=tokens)
    blk = bf16_to_f32(x_a_bf16[out["tokens"]]).astype(np.float64) + out["out_f64"]
    out.update(xn=xn, block_f32=blk.astype(np.float32), block_bf16=f32_to_bf16(blk.astype(np.float32)))
    return out
