/* mote.h -- C ABI of the MI355X (gfx950) MoTE-layer forward library.
 *
 * One MoTE layer (Mixture of Ternary Experts, arXiv 2506.14435, Section 3.1) is
 *     out = FFN(x) + MoE(x)                                   (Eq.2 without residual and LN)
 *     MoE(x) = sum_{i in top-k} P(x)_i * FFN^T_i(x)            (Eq.3, Eq.4, sparse gate)
 *     FFN^T_i(x) = Q_w(W_down) Q_a(h),  h = Q_w(W_up) Q_a(x) (*) SiLU(Q_w(W_gate) Q_a(x))   (Eq.5-6)
 *     Q_w: absmean ternary {-1,0,1} with one scale per matrix, Q_a: per-token absmax int8     (Eq.7-10)
 * FFN is the full-precision (bf16) shared SwiGLU expert; the routed experts are stored as
 * 2-bit codes (INT2 storage, end of Section 3.1) and contracted on int8 MFMA with int32
 * accumulation.
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer into memory the CALLER owns, 16-byte aligned.
 *     The library never allocates or frees device memory and never synchronises inside these
 *     calls; all work is ordered on the HIP stream passed as `hip_stream` (a hipStream_t cast
 *     to void*, NULL is the default stream).  For batches where it pays, mote_layer_forward
 *     runs the shared expert on a helper stream of its own (created on first use, default
 *     priority) that it forks from and joins back into `hip_stream` with events, so to the
 *     caller the call behaves like work on `hip_stream` alone; mote_tuning_set(MOTE_KNOB_NO_FORK, 1)
 *     keeps everything on one stream.  The library reads no environment variable.  Host-side
 *     state (helper stream, timing events, knobs) is not thread-safe.
 *     Inputs and outputs must not alias.
 *   - Matrices are row-major.  A weight matrix is [n_out, n_in] and acts on a column
 *     vector of n_in channels (Section 3.1, sentence after Eq.10).
 *   - bf16 data is the raw 16-bit pattern.
 *   - Errors are return codes.  Shapes are validated before anything is enqueued; on an
 *     error nothing has been launched unless the code is MOTE_ERR_HIP.
 *   - There is no CPU fallback: without a gfx950 device every call fails with MOTE_ERR_HIP.
 */
#ifndef MOTE_H
#define MOTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOTE_OK = 0,
  MOTE_ERR_INVALID_ARG = 1,        /* null pointer, negative size, bad enum            */
  MOTE_ERR_UNSUPPORTED_SHAPE = 2,  /* violates the shape limits listed per entry point */
  MOTE_ERR_WORKSPACE_TOO_SMALL = 3,
  MOTE_ERR_HIP = 4                 /* a HIP launch / runtime call failed               */
} mote_status;

/* Static, NUL-terminated description of a status code (host memory, never freed). */
const char* mote_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int mote_version(void);

/* ---------------------------------------------------------------------------------------
 * Q_w + INT2 pack  (Eq.7, Eq.9, Eq.10; INT2 storage of the ternary weights, end of
 * Section 3.1).  Offline, once per weight matrix.
 *
 *   alpha  = max( fp32( sum|W| (fp64) / (n_out*n_in) ), 1e-5 )
 *   t      = clip( round_half_even( W / alpha ), -1, 1 )           (fp32 IEEE divide)
 *   code   = t + 1  in {0,1,2}; code 3 is never written
 *
 * Packed layout (this library's; the paper fixes none): tiles of 32 rows x 128 input
 * channels, tile (nt, kt) at 32-bit word offset 256*(nt*(n_in/128) + kt).  In a tile, word
 * 4*(32*g + r) + s (r = row%32, g in {0,1}, s in 0..3) holds the codes of row 32*nt + r for
 * channels 128*kt + 32*s + 16*g + i, i = 0..15, code i at bit 8*(i%4) + 2*(i/4).  Hence a
 * 64-lane wavefront fetches a tile with one 16-byte load per lane, and (word >> 2j) &
 * 0x03030303, j = 0..3, are four int8 MFMA operand registers in channel order.
 */
enum { MOTE_DTYPE_F32 = 0, MOTE_DTYPE_BF16 = 1 };

/* Bytes of the packed form of an [n_out, n_in] matrix: n_out*n_in/4. */
size_t mote_packed_bytes(int64_t n_out, int64_t n_in);

/* w       in : device, [n_out, n_in] latent weights, fp32 or bf16 (w_dtype)
 * packed  out: device, mote_packed_bytes(n_out, n_in) bytes (also used as scratch for the
 *              partial sums of the reduction before it is overwritten)
 * alpha   out: device, 1 float, the clamped scale
 * Limits: n_out % 32 == 0, n_in % 128 == 0, both > 0. */
mote_status mote_pack_ternary(const void* w, int w_dtype, int64_t n_out, int64_t n_in,
                              uint32_t* packed, float* alpha, void* hip_stream);

/* The 1-bit weight quantiser of the routed-expert ablation (Section 4.4, Table 5: binary weight
 * network): t = sign(W) with sign(0) = +1, alpha as above.  The codes t + 1 in {0, 2} use the same
 * 2-bit container, so binary experts run through mote_layer_forward unchanged (a 1-bit container
 * is not provided).  Arguments and limits as mote_pack_ternary. */
mote_status mote_pack_binary(const void* w, int w_dtype, int64_t n_out, int64_t n_in,
                             uint32_t* packed, float* alpha, void* hip_stream);

/* ---------------------------------------------------------------------------------------
 * Round-to-nearest INT8 / INT4 quantisation of a shared-expert matrix (Section 4.3, Table 3).
 * The paper names the method only; this library's reading: weight-only, symmetric, one scale
 * per output channel,
 *   s_n = max(max_c |W[n,c]|, 1e-5) / qmax            (fp32 divide; qmax = 127 or 7)
 *   q   = clip(round_half_even(W[n,c] / s_n), -qmax, qmax)   (fp32 divide)
 * Storage: row-major over output rows, n_in*bits/8 bytes per row, two's-complement bytes (INT8)
 * or nibbles (INT4; position p of a row in byte p/2, bits 4*(p%2)..+3), channels permuted inside
 * groups: INT8 groups of 32, position 16g + 8a + i holds channel 16a + 8g + i; INT4 groups of 64,
 * position 32g + 8s + i holds channel 16s + 8g + i (g, a in {0,1}, s in 0..3, i in 0..7), so that
 * the 16 bytes a lane reads are its operands of consecutive 32x32x16 MFMAs.
 *
 * w      in : device bf16 [n_out, n_in]
 * packed out: device, mote_rtn_packed_bytes(n_out, n_in, bits) bytes
 * scales out: device fp32 [n_out]
 * Limits: bits in {8, 4}; n_out % 32 == 0, n_in % 128 == 0. */
size_t mote_rtn_packed_bytes(int64_t n_out, int64_t n_in, int bits);
mote_status mote_pack_rtn(const void* w, int64_t n_out, int64_t n_in, int bits, void* packed,
                          float* scales, void* hip_stream);

/* ---------------------------------------------------------------------------------------
 * Straight-through estimator of Section 3.2 (quantisation-aware training) for one grouped ternary
 * linear layer of Section 3.1, Y_e = Q_a(X_e) Q_w(W_e)^T, rows grouped by expert: the gradients
 * treat both quantisers as the identity, dL/dW = dL/dQ_w(W) and dL/dX = dL/dQ_a(X), i.e.
 *
 *   dx[r, c]    = alpha_e * sum_n dy[r, n] * t_e[n, c]                         (r a row of expert e)
 *   dw[e][n, c] = sum_{r in e} bf16(dy[r, n] * (beta[r] / 127)) * q[r, c]
 *
 * bf16 operands (ternary values and int8 codes are exact in bf16), fp32 accumulation on the bf16
 * MFMA; the activation scale beta[r] / 127 (one fp32 divide) is folded into the gradient row
 * with one fp32 multiply and one rounding to bf16, because dw contracts over r.
 *
 * dy           in : bf16 [R, N], row r belongs to expert e for offsets[e] <= r < offsets[e+1]
 * offsets_host in : HOST int32 [E + 1], ascending, offsets[0] = 0, offsets[E] = R (the expert
 *                   counts of the forward pass, read back by the caller)
 * packed       in : E packed ternary matrices [N, K] back to back (mote_pack_ternary)
 * alpha        in : fp32, alpha of expert e at alpha[e * alpha_stride]
 * q, beta      in : Q_a(X): int8 [R, K] and the clamped absmax fp32 [R] of each row
 * dx           out: fp32 [R, K]
 * dw           out: fp32 [E, N, K] (zero for an expert without rows)
 * workspace       : device, >= mote_ste_backward_workspace_bytes(R, N, K, E) bytes, 256-byte aligned
 *                   (the transposed ternary weights of all experts as bf16, at most 4 GiB of them at a
 *                   time, the transposed gradient rows and codes, partial sums of dx: about
 *                   2 E N K + 2 R (N + K) + 32 R K bytes)
 * Limits: N % 128 == 0, K % 128 == 0, 1 <= E <= 64, R >= 0; every operand of one expert below
 * 2 GiB.  Enqueued on hip_stream; the host array is read before the call returns.
 * Returns MOTE_ERR_INVALID_ARG for NULL pointers or offsets that are not ascending from 0 to R,
 * MOTE_ERR_UNSUPPORTED_SHAPE, MOTE_ERR_WORKSPACE_TOO_SMALL, MOTE_ERR_HIP. */
size_t mote_ste_backward_workspace_bytes(int R, int N, int K, int E);
mote_status mote_ste_linear_backward(const void* dy, const int32_t* offsets_host, const uint32_t* packed,
                                     const float* alpha, int alpha_stride, const int8_t* q, const float* beta,
                                     int R, int N, int K, int E, float* dx, float* dw, void* workspace,
                                     size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------
 * Router: gate softmax of Eq.3 and GShard-style top-k selection (Section 3.1; Section 4.1
 * uses top-1 routing).
 *
 *   logits[t,e] = sum_c x[t,c] * w_router[c,e] (+ router_bias[e]),   fp64 accumulation
 *   P = softmax over all E logits; the k largest logits are selected, in descending order,
 *   exact ties to the lower expert index; topk_p = P[selected], NOT renormalised (Eq.4
 *   multiplies by P(x)_i itself).
 *
 * x            in : bf16 [T, d]
 * w_router     in : bf16 [d, E]   (the router projection stays BF16, Section 3.1)
 * router_bias  in : fp32 [E] or NULL.  NULL is the paper's layer; the bias only serves
 *                   synthetic workloads that need a prescribed expert load.
 * topk_idx     out: int32 [T, k]
 * topk_p       out: fp32  [T, k]
 * expert_counts out: int32 [E] or NULL; number of (token, slot) pairs routed to each expert
 * Limits: d % 128 == 0, 1 <= E <= 64, 1 <= k <= min(E, 8), T >= 0 (T == 0 is a no-op). */
mote_status mote_router_topk(const void* x, const void* w_router, const float* router_bias,
                             int T, int d, int E, int k, int32_t* topk_idx, float* topk_p,
                             int32_t* expert_counts, void* hip_stream);

/* Router plus the load-balancing statistic of Section 3.3 (Eq.12, following Switch
 * Transformers):  loss = E/|X| * sum_i t_i * sum_x P(x)_i, t_i = number of (token, slot) pairs
 * routed to expert i, exactly as printed (the cited work divides by |X| once more: loss / T).
 * Outputs beyond mote_router_topk (all required): expert_counts int32 [E] = t_i, gate_p fp32 [T, E]
 * = the whole gate distribution, gate_p_sum fp32 [E] = sum_x P(x)_i (fp64 sums in a fixed order),
 * loss fp32 [1].  T >= 1. */
mote_status mote_router_balance(const void* x, const void* w_router, const float* router_bias,
                                int T, int d, int E, int k, int32_t* topk_idx, float* topk_p,
                                int32_t* expert_counts, float* gate_p, float* gate_p_sum, float* loss,
                                void* hip_stream);

/* ---------------------------------------------------------------------------------------
 * Whole layer.
 */
typedef struct {
  int d_model, d_ff_shared, d_ff_routed, n_experts, top_k;
  const void* w_router;        /* bf16 [d, E]                                             */
  const float* router_bias;    /* fp32 [E] or NULL                                        */
  const void* ws_gate;         /* shared expert, bf16 [F_s, d]                            */
  const void* ws_up;           /* bf16 [F_s, d]                                           */
  const void* ws_down;         /* bf16 [d, F_s]                                           */
  const uint32_t* wt_gate;     /* routed, packed: E matrices [F_r, d], expert-major       */
  const uint32_t* wt_up;       /* E matrices [F_r, d]                                     */
  const uint32_t* wt_down;     /* E matrices [d, F_r]                                     */
  const float* alpha;          /* fp32 [E, 3]: (gate, up, down) scale of each expert      */
  /* Post-training quantised shared expert (Section 4.3, Table 3).  shared_bits == 0: ws_* are bf16
   * (the paper's layer).  8 or 4: ws_* point at the packed codes written by mote_pack_rtn and
   * ss_* at their fp32 row scales ([F_s], [F_s], [d]); activations stay bf16. */
  int shared_bits;
  const float* ss_gate;
  const float* ss_up;
  const float* ss_down;
} mote_layer;

/* Optional copies of the intermediates, for stage-wise parity checks.  Every member may be
 * NULL.  R = T*k routed rows in dispatch order: grouped by expert (ascending), inside an
 * expert by flat position t*k + j (ascending). */
typedef struct {
  int32_t* topk_idx;   /* [T, k]                                                          */
  float* topk_p;       /* [T, k]                                                          */
  int32_t* counts;     /* [E]                                                             */
  int32_t* row_of;     /* [T, k]  dispatch row of (t, j)                                  */
  int32_t* tok_of;     /* [R]     token of a dispatch row                                 */
  int8_t* q_x;         /* [T, d]  Q_a(x) integers                                         */
  float* beta_x;       /* [T]     clamped absmax of x                                     */
  int32_t* acc_gate;   /* [R, F_r] integer contraction t_gate . q_x                       */
  int32_t* acc_up;     /* [R, F_r]                                                        */
  uint16_t* h;         /* [R, F_r] bf16 hidden activation of the routed experts           */
  int8_t* q_h;         /* [R, F_r] Q_a(h) integers                                        */
  float* beta_h;       /* [R]                                                             */
  int32_t* acc_down;   /* [R, d]  integer contraction t_down . q_h                        */
  uint16_t* h_s;       /* [T, F_s] bf16 hidden activation of the shared expert            */
  float* y_s;          /* [T, d]  shared expert output                                    */
  float* out_f32;      /* [T, d]  layer output before the final bf16 rounding             */
  uint16_t* xn;        /* [T, d]  LN(x^a), written by mote_block_forward only             */
} mote_taps;

/* Bytes of scratch that serve mote_layer_forward for every batch of 1..T_max tokens (0 on a bad
 * shape): the largest layout over those batch sizes (the kernel family and the number of K-split
 * partial planes depend on the batch size, not monotonically). */
size_t mote_layer_workspace_bytes(const mote_layer* layer, int T_max);

/* out = FFN(x) + MoE(x)  (Eq.2 + Eq.4; no residual add, no LayerNorm).
 * x    in : bf16 [T, d]
 * out  out: bf16 [T, d]
 * workspace: device scratch of at least mote_layer_workspace_bytes(layer, T) bytes, 256-byte
 *            aligned; contents are undefined afterwards; calls sharing a workspace must be
 *            ordered on one stream.
 * taps : NULL in production.
 * Limits: d, F_s, F_r % 128 == 0; 1 <= E <= 64; 1 <= k <= min(E, 8); 0 <= T; T*k < 2^24;
 *         T*d, T*F_s and T*k*F_r below 2^31 (32-bit byte offsets inside the kernels). */
mote_status mote_layer_forward(const mote_layer* layer, const void* x, int T, void* out,
                               void* workspace, size_t workspace_bytes, const mote_taps* taps,
                               void* hip_stream);

/* The MoE half of a block, Eq.2:  out = x^a + MoE(LN(x^a)) + FFN(LN(x^a)).
 * LN is the base model's normalisation: RMSNorm for the Qwen2.5 models the paper up-cycles
 * (y = x / sqrt(mean x^2 + eps) * gamma), or layer normalisation taken literally
 * (y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance).  Statistics in fp64; LN(x^a)
 * is rounded once to bf16 (it is the bf16 hidden state the layer of Section 3.1 acts on); the
 * residual x^a is added in fp32 before the single bf16 rounding of the output.
 * gamma, beta: device bf16 [d] (beta only for MOTE_NORM_LAYER).  Everything else as in
 * mote_layer_forward, including the workspace size. */
enum { MOTE_NORM_RMS = 1, MOTE_NORM_LAYER = 2 };
typedef struct {
  int kind;            /* MOTE_NORM_RMS or MOTE_NORM_LAYER */
  const void* gamma;   /* bf16 [d] */
  const void* beta;    /* bf16 [d], MOTE_NORM_LAYER only */
  double eps;
} mote_norm;
mote_status mote_block_forward(const mote_layer* layer, const mote_norm* norm, const void* x_a, int T, void* out,
                               void* workspace, size_t workspace_bytes, const mote_taps* taps,
                               void* hip_stream);

/* The same forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch is a
 * static device array of the library, MOTE_STATIC_WORKSPACE_BYTES per GPU, held from the time the
 * library is loaded until the process ends.  The call allocates and frees nothing (no device
 * memory, no stream, no event): every kernel, the shared expert included, runs on `hip_stream`,
 * and stage timing does not apply.  Arguments, limits and results are those of
 * mote_layer_forward (the results are bit-identical).  A batch whose layout needs more than the
 * array (mote_layer_workspace_bytes(layer, T) > MOTE_STATIC_WORKSPACE_BYTES) is refused with
 * MOTE_ERR_WORKSPACE_TOO_SMALL before anything is launched; 64 MiB serve the 3B-width layer
 * (d = 2048, F = 11008, 16 experts, top-2) up to 256 tokens and the 7B width up to 128.  All calls
 * on one GPU share that GPU's array, which keeps the previous call's contents: calls must be
 * ordered on one stream (or otherwise not overlap), two that overlap on one GPU race. */
#define MOTE_STATIC_WORKSPACE_BYTES (64u << 20)
mote_status mote_layer_forward_static(const mote_layer* layer, const void* x, int T, void* out,
                                      const mote_taps* taps, void* hip_stream);

/* ---------------------------------------------------------------------------------------
 * Measurement support (not part of the layer's mathematics).
 */
enum {
  MOTE_STAGE_ROUTER_QUANT = 0, /* router + softmax/top-k + Q_a(x)                 */
  MOTE_STAGE_DISPATCH = 1,     /* counts, offsets, permutation, tile list         */
  MOTE_STAGE_ROUTED_GATE_UP = 2,
  MOTE_STAGE_QUANT_H = 3,
  MOTE_STAGE_ROUTED_DOWN = 4,
  MOTE_STAGE_SHARED_GATE_UP = 5,
  MOTE_STAGE_SHARED_DOWN = 6,
  MOTE_STAGE_COMBINE = 7,
  MOTE_N_STAGES = 8
};

/* enable != 0: every following mote_layer_forward brackets each stage with HIP events on
 * the caller's stream (created on first use, host-side state, not thread-safe). */
mote_status mote_stage_timing(int enable);

/* Waits for the last timed forward and writes the MOTE_N_STAGES stage durations in
 * milliseconds to host memory `ms`; a stage that did not run reports 0. */
mote_status mote_stage_times(float* ms_host);

/* Milliseconds that two consecutive event records on `hip_stream` read with nothing between them
 * (median of 33 pairs; synchronises with the stream).  A stage time of mote_stage_times is the
 * stage's kernel plus this much, which matters for kernels of a few tens of microseconds. */
mote_status mote_event_pair_overhead(float* ms_host, void* hip_stream);

/* Tuning knobs for experiments (the defaults are what the measurements chose; the library reads
 * nothing from the environment).  Host-side state, not thread-safe.  Some knobs change the
 * workspace layout: set them before mote_layer_workspace_bytes and keep them until the forwards
 * that use that workspace have been enqueued. */
enum {
  MOTE_KNOB_NO_FORK = 0,             /* 1: shared expert on the caller's stream (default 0)            */
  MOTE_KNOB_FORK_MIN_LOG2 = 1,       /* log2 of T*d*F_s from which the forward forks (29)              */
  MOTE_KNOB_EVENT_FENCE = 2,         /* 1: fork/join events with a system-scope fence; before the first
                                        forked forward (0)                                             */
  MOTE_KNOB_QUANT_WIDE = 3,          /* 1: 256-thread row quantiser for every row length (0)           */
  MOTE_KNOB_ROUTED_VARIANT = 4,      /* tile configuration of the large-batch routed gate-up GEMM (0)  */
  MOTE_KNOB_ROUTED_DOWN_VARIANT = 5, /* ... of the routed down GEMM (-1: as gate-up)                   */
  MOTE_KNOB_SHARED_VARIANT = 6,      /* ... of the shared GEMMs (0: chosen by shape)                   */
  MOTE_KNOB_GROUP_M = 7,             /* row tiles per band of the tile order (2)                       */
  MOTE_KNOB_DYNAMIC_ROUNDS = 8,      /* tiles per workgroup from which tiles are drawn (4)             */
  MOTE_KNOB_DECODE_VARIANT = 9,      /* routed decode kernel: 0 K-split, 1 / 2 wave-streaming with two
                                        workgroups of four / one of eight wavefronts per CU (-1: by shape) */
  MOTE_KNOB_ROUTER_TOKEN_BLOCKS = 10,/* largest T with one token per router workgroup (256)            */
  MOTE_KNOB_DOWN_SPLIT_TILES = 11,   /* routed down projection: two K planes while it has fewer
                                        128 x 128 output tiles than this (600)                         */
  MOTE_KNOB_MID_ROWS_LO = 12,        /* 64-row plan tiles (wave-streaming kernel) when an expert sees on
                                        average more than this many rows (31) ...                      */
  MOTE_KNOB_MID_ROWS_HI = 13,        /* ... and at most this many (60); lo >= hi switches them off     */
  MOTE_KNOB_STE_BATCH_MIB = 14,      /* mote_ste_linear_backward: the experts of one grouped dX GEMM have at
                                        most this many MiB of expanded weights together, 1 .. 4095 (4095);
                                        mote_ste_backward_workspace_bytes depends on it                 */
  MOTE_N_KNOBS = 15
};
mote_status mote_tuning_set(int knob, int value);

/* dst[i] = src[i] for n_bytes (multiple of 16) with a plain grid-stride copy kernel: the
 * known-size transfer used to calibrate HBM byte counters. */
mote_status mote_calib_copy(void* dst, const void* src, size_t n_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOTE_H */
