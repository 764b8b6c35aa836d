// Host-side launch functions of the kernel translation units (internal, C++).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mote {

// Tuning knobs (experiments only; set through mote_tuning_set, never read from the environment).
// The values are plain ints in one table of mote_api.hip; -1 means "the library's own choice".
enum Knob {
  kKnobNoFork = 0,           // 1: shared expert on the caller's stream
  kKnobForkMinLog2,          // log2 of T*d*F_s from which the forward forks
  kKnobEventFence,           // 1: fork / join events carry a system-scope fence
  kKnobQuantWide,            // 1: 256-thread row quantiser for every row length
  kKnobRoutedVariant,        // tile configuration of the large-batch routed gate-up GEMM
  kKnobRoutedDownVariant,    // ... of the routed down GEMM (-1: same as gate-up)
  kKnobSharedVariant,        // ... of the shared GEMMs (0: by shape)
  kKnobGroupM,               // row tiles per band of the tile order
  kKnobDynamicRounds,        // tiles per workgroup from which tiles are drawn
  kKnobDecodeVariant,        // routed decode kernel: 0 K-split, 1 / 2 wave-streaming with 4 / 8 wavefronts per workgroup
  kKnobRouterTokenBlocks,    // largest T with one token per router workgroup
  kKnobDownSplitTiles,       // routed down projection: two K planes while there are fewer 128 x 128 output tiles than this
  kKnobMidRowsLo,            // 64-row plan tiles for more than this many rows per expert on average ...
  kKnobMidRowsHi,            // ... and at most this many
  kKnobSteBatchMiB,          // expanded weights (MiB) of the experts that share one grouped dX GEMM
  kKnobCount
};
int knob(int id);

// binary: the 1-bit quantiser t = sign(w) (sign(0) = +1) instead of the ternary RoundClip
hipError_t launch_pack_ternary(const void* w, bool is_bf16, int64_t n_out, int64_t n_in, uint32_t* packed,
                               float* alpha, bool binary, hipStream_t stream);

// Router (Eq.3 + top-k) fused with Q_a(x) (Eq.8).  q_x / beta_x / rowsum_x may be null
// (router only).
hipError_t launch_router_quant(const uint16_t* x, const uint16_t* w_router, const float* bias, int T, int d,
                               int E, int k, int32_t* topk_idx, float* topk_p, int8_t* q_x, float* beta_x,
                               int32_t* rowsum_x, float* gate_p, hipStream_t stream);   // gate_p: optional fp32 [T, E], the whole softmax

hipError_t launch_expert_counts(const int32_t* topk_idx, int R, int E, int32_t* counts, hipStream_t stream);

// Dispatch plan: counts, offsets, row_of / tok_of (expert-major, stable) and the list of
// row tiles (tile_m rows each) that the grouped GEMMs walk.
struct DispatchPlan {
  int32_t* counts;      // [E]
  int32_t* offsets;     // [E+1]
  int32_t* row_of;      // [T*k]
  int32_t* tok_of;      // [T*k]
  int32_t* tile_expert; // [max_tiles]
  int32_t* tile_row0;   // [max_tiles]
  int32_t* tile_rows;   // [max_tiles]
  int32_t* n_tiles;     // [1]
  int32_t* row_planes;  // [T*k] per dispatch row: 2 bits per channel tile of the down projection, partial planes - 1 of its accumulators
  int32_t* sched;       // [16 * kSchedStride] tile counters of the two grouped GEMMs (8 lists each, one cache line per counter), zeroed with the plan
};
constexpr int kSchedStride = 32;   // ints between two counters
constexpr int kSplitMaxPlanes = 4;  // K planes a pair of the last round of the down projection may be cut into
hipError_t launch_dispatch_plan(const int32_t* topk_idx, int T, int k, int E, int tile_m, const DispatchPlan& plan,
                                hipStream_t stream);

// Grouped ternary GEMMs over the dispatch plan.
struct RoutedGemmArgs {
  const int8_t* q;          // activation rows [*, K] int8
  const int32_t* gather;    // dispatch row -> row of q / beta / rowsum, or null for identity
  const float* beta;        // clamped absmax per row of q
  const int32_t* rowsum;    // sum of the int8 row (zero-point correction of code = t + 1)
  const uint32_t* w_gate;   // packed, expert-major (gate / down)
  const uint32_t* w_up;     // packed (gate-up mode only)
  const float* alpha;       // [E, 3]
  DispatchPlan plan;
  int max_tiles;            // upper bound on *plan.n_tiles known on the host
  int tile_m;               // rows per plan tile
  int K, N;                 // contraction length, output width (per matrix)
  int64_t q_rows;           // rows of q (q_rows * K <= 2^31: 32-bit buffer offsets)
  int64_t out_rows;         // rows of the output (dispatch rows R)
  uint16_t* h;              // gate-up: bf16 [R, N]
  int32_t* acc_out;         // down: int32 [R, N] (decode: partial planes [planes][R, N])
  int64_t partial_stride;   // elements between partial planes (down projections)
  int planes;               // K planes of the large-batch down projection (1: none)
  int split_max;            // planes a pair of the last round may be cut into (down projection with planes == 1; <= 1: never)
  int32_t* tap_gate;        // optional int32 [R, N]
  int32_t* tap_up;
};
hipError_t launch_routed_gate_up(const RoutedGemmArgs& a, hipStream_t stream);
hipError_t launch_routed_down(const RoutedGemmArgs& a, hipStream_t stream);
int routed_down_tile_n(int planes);
int routed_down_planes(int T, int k, int E, int d, int F);   // large-batch down: K planes for a shape
int shared_down_planes(int T, int d, int F);
int tile_group_m();                      // row tiles per band of the large-batch tile order
int routed_tile_m(int T, int k, int E, int d, int F);  // plan tile size chosen for a workload (32, 64: decode kernels)
bool routed_mid_kernel_fits(int d, int F);             // the 64-row wave-streaming kernel serves this shape

// Decode (small batch) variants: weights streamed once, K split across wavefronts and, for the
// down projections, across workgroups into partial planes that the combine kernel adds.
hipError_t launch_routed_decode_gate_up(const RoutedGemmArgs& a, hipStream_t stream);
hipError_t launch_routed_decode_down(const RoutedGemmArgs& a, hipStream_t stream);
int routed_decode_down_planes(int K);
constexpr int kSharedDecodeMaxTokens = 64;
hipError_t launch_shared_decode_gate_up(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up, int T, int d,
                                        int F, uint16_t* h_s, hipStream_t stream);
hipError_t launch_shared_decode_down(const uint16_t* h_s, const uint16_t* w_down, int T, int d, int F, float* y_s,
                                     hipStream_t stream);
int shared_decode_down_planes(int d, int K);

// Q_a(h): per dispatch row absmax int8 of the bf16 hidden activation.
hipError_t launch_quant_rows(const uint16_t* h, int rows, int F, int8_t* q, float* beta, int32_t* rowsum,
                             hipStream_t stream);

// Shared expert (bf16 MFMA, fp32 accumulation).
hipError_t launch_shared_gate_up(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up, int T, int d,
                                 int F, uint16_t* h_s, hipStream_t stream);
hipError_t launch_shared_down(const uint16_t* h_s, const uint16_t* w_down, int T, int d, int F, float* y_s,
                              hipStream_t stream);
// The same GEMMs with a per-output-channel scale applied to the fp32 sums (integer-valued bf16
// weights of an RTN-quantised shared expert); scales may be null.
hipError_t launch_shared_gate_up_scaled(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up,
                                        const float* s_gate, const float* s_up, int T, int d, int F, uint16_t* h_s,
                                        hipStream_t stream);
hipError_t launch_shared_down_scaled(const uint16_t* h_s, const uint16_t* w_down, const float* s_down, int T, int d,
                                     int F, float* y_s, hipStream_t stream);
// RTN-quantised shared expert, decode (T <= kSharedDecodeMaxTokens): packed INT8 / INT4 codes
hipError_t launch_shared_q_decode_gate_up(const uint16_t* x, const void* w_gate, const void* w_up, const float* s_gate,
                                          const float* s_up, int bits, int T, int d, int F, uint16_t* h_s,
                                          hipStream_t stream);
hipError_t launch_shared_q_decode_down(const uint16_t* h_s, const void* w_down, const float* s_down, int bits, int T,
                                       int d, int F, float* y_s, hipStream_t stream);
hipError_t launch_rtn_pack(const uint16_t* w, int64_t n_out, int64_t n_in, int bits, void* packed, float* scales,
                           hipStream_t stream);
hipError_t launch_rtn_dequant(const void* packed, int64_t n_out, int64_t n_in, int bits, uint16_t* out, hipStream_t stream);
// LN(.) of Eq.1-2: kind 1 RMSNorm, kind 2 layer normalisation (beta used by kind 2 only)
hipError_t launch_norm_rows(const uint16_t* x, const uint16_t* gamma, const uint16_t* beta, int kind, double eps, int T,
                            int d, uint16_t* y, hipStream_t stream);
// Eq.12 from the gate probabilities [T, E] and the routed counts [E]
hipError_t launch_balance(const float* gate_p, const int32_t* counts, int T, int E, float* gate_p_sum, float* loss,
                          hipStream_t stream);

// out = bf16( y_s + sum_j p[t,j] * (acc_down[row_of[t,j]] * (beta_h/127 * alpha_down)) ).
// y_s and acc_down may come as several partial planes (decode K splits), added in plane order.
struct CombineArgs {
  const float* y_s; int y_planes; int64_t y_stride;
  const int32_t* acc_down; int d_planes; int64_t d_stride;
  const int32_t* row_planes;   // plan.row_planes, or null: d_planes for every row and channel
  int d_tile_n;                // channels per channel tile of row_planes
  const float* beta_h; const float* alpha;
  const int32_t* topk_idx; const float* topk_p; const int32_t* row_of;
  int T, d, k;
  const uint16_t* residual;   // optional bf16 [T, d] added before the final rounding (x^a of Eq.2)
  uint16_t* out;
  float* out_f32;         // optional taps
  float* tap_y_s;         // [T, d] summed shared output
  int32_t* tap_acc_down;  // [R, d] summed down accumulators
};
hipError_t launch_combine(const CombineArgs& a, hipStream_t stream);

// bf16 GEMMs of two row-major operands contracted along their rows, fp32 output (shared_ffn.hip):
// the contraction cut into K ranges given by a host table, one output plane per range
hipError_t launch_gemm_tn_f32_kgroups(const uint16_t* act, const uint16_t* w, int M, int N, const int32_t* k0_host,
                                      int n_groups, float* out, hipStream_t stream);
// groups of rows with a weight matrix (and scale vector) each; row0_host: host int32 [n_groups + 1]
int grouped_gemm_planes(const int32_t* row0_host, int n_groups, int N, int K, int max_planes);
hipError_t launch_gemm_grouped_f32(const uint16_t* act, const uint16_t* w, const int32_t* row0_host, int n_groups, int N,
                                   int K, float* out, const float* scale, int planes, hipStream_t stream);
// straight-through gradients of a grouped ternary linear layer (ste_backward.hip); offsets_host: host int32 [E + 1]
size_t ste_backward_workspace_bytes(int R, int N, int K, int E);
hipError_t launch_ste_backward(const uint16_t* dy, const int32_t* offsets_host, const uint32_t* packed, const float* alpha,
                               int alpha_stride, const int8_t* q, const float* beta, int R, int N, int K, int E,
                               float* dx, float* dw, void* workspace, hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t stream);

}  // namespace mote
