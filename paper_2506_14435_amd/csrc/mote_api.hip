// C ABI of the MoTE-layer library: argument validation, workspace carving and the
// sequence of kernel launches for one forward pass (Eq.2-10 of Section 3.1).
#include "../../include/mote.h"

#include <hip/hip_runtime.h>

#include "launch.h"
#include <algorithm>

namespace mote {
// Tuning knobs: defaults are what the measurements chose; mote_tuning_set overwrites them.
static int g_knobs[kKnobCount] = {
    /* NoFork */ 0, /* ForkMinLog2 */ 29, /* EventFence */ 0, /* QuantWide */ 0, /* RoutedVariant */ 0,
    /* RoutedDownVariant */ -1, /* SharedVariant */ 0, /* GroupM */ 2, /* DynamicRounds */ 4,
    /* DecodeVariant */ -1, /* RouterTokenBlocks */ 256, /* DownSplitTiles */ 600, /* MidRowsLo */ 31,
    /* MidRowsHi */ 60, /* SteBatchMiB */ 4095};
int knob(int id) { return (id >= 0 && id < kKnobCount) ? g_knobs[id] : -1; }
}  // namespace mote

namespace {

using namespace mote;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Workspace {
  // dispatch
  int32_t* topk_idx; float* topk_p; int32_t* counts; int32_t* offsets; int32_t* n_tiles; int32_t* sched; int32_t* row_planes;
  int32_t* row_of; int32_t* tok_of; int32_t* tile_expert; int32_t* tile_row0; int32_t* tile_rows;
  // Q_a(x)
  int8_t* q_x; float* beta_x; int32_t* rs_x;
  // routed experts
  uint16_t* h; int8_t* q_h; float* beta_h; int32_t* rs_h; int32_t* acc_down;
  // shared expert
  uint16_t* h_s; float* y_s;
  uint16_t* deq_gate; uint16_t* deq_up; uint16_t* deq_down;   // integer-valued bf16 copies of RTN weights (large batches)
  // block prologue
  uint16_t* xn;      // LN(x^a), bf16 [T, d]
  size_t bytes;
  int max_tiles;
  int tile_m;        // 32, 64: decode kernels, 128: large-batch kernels
  int d_planes;      // uniform partial planes of the routed down accumulators
  int d_split;       // planes a tile of the last round may be cut into instead (large batch, d_planes == 1)
  int y_planes;      // partial planes of the shared expert output
};

// Kernels address activations with 32-bit byte offsets.
bool batch_ok(const mote_layer* l, int T) {
  const int64_t lim = int64_t{1} << 31;
  const int64_t R = static_cast<int64_t>(T) * l->top_k;
  return R < (1 << 24) && static_cast<int64_t>(T) * l->d_model < lim && R * l->d_ff_routed < lim &&
         static_cast<int64_t>(T) * l->d_ff_shared < lim;
}

bool layer_shape_ok(const mote_layer* l) {
  if (l->d_model <= 0 || l->d_ff_shared <= 0 || l->d_ff_routed <= 0) return false;
  if (l->d_model % 128 || l->d_ff_shared % 128 || l->d_ff_routed % 128) return false;
  if (l->n_experts < 1 || l->n_experts > 64) return false;
  if (l->top_k < 1 || l->top_k > l->n_experts || l->top_k > 8) return false;
  if (l->shared_bits != 0 && l->shared_bits != 8 && l->shared_bits != 4) return false;
  return true;
}

// Carves the workspace; with base == nullptr only the size is computed.
Workspace carve(const mote_layer* l, int T, char* base) {
  Workspace w{};
  size_t off = 0;
  auto take = [&](size_t bytes) -> char* {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes ? bytes : 1);
    return p;
  };
  const size_t R = static_cast<size_t>(T) * l->top_k;
  const size_t d = l->d_model, Fr = l->d_ff_routed, Fs = l->d_ff_shared;
  w.max_tiles = static_cast<int>(R / 32 + l->n_experts);
  w.tile_m = routed_tile_m(T, l->top_k, l->n_experts, l->d_model, l->d_ff_routed);
  w.d_planes = w.tile_m != 128 ? routed_decode_down_planes(l->d_ff_routed)
                              : routed_down_planes(T, l->top_k, l->n_experts, l->d_model, l->d_ff_routed);
  w.d_split = (w.tile_m == 128 && w.d_planes == 1) ? kSplitMaxPlanes : 1;
  w.y_planes = T <= kSharedDecodeMaxTokens ? shared_decode_down_planes(l->d_model, l->d_ff_shared)
                                           : shared_down_planes(T, l->d_model, l->d_ff_shared);
  w.topk_idx = reinterpret_cast<int32_t*>(take(R * 4));
  w.topk_p = reinterpret_cast<float*>(take(R * 4));
  w.counts = reinterpret_cast<int32_t*>(take(64 * 4));
  w.offsets = reinterpret_cast<int32_t*>(take(65 * 4));
  w.n_tiles = reinterpret_cast<int32_t*>(take(4));
  w.sched = reinterpret_cast<int32_t*>(take(16 * kSchedStride * 4));
  w.row_planes = reinterpret_cast<int32_t*>(take(R * 4));
  w.row_of = reinterpret_cast<int32_t*>(take(R * 4));
  w.tok_of = reinterpret_cast<int32_t*>(take(R * 4));
  w.tile_expert = reinterpret_cast<int32_t*>(take(static_cast<size_t>(w.max_tiles) * 4));
  w.tile_row0 = reinterpret_cast<int32_t*>(take(static_cast<size_t>(w.max_tiles) * 4));
  w.tile_rows = reinterpret_cast<int32_t*>(take(static_cast<size_t>(w.max_tiles) * 4));
  w.q_x = reinterpret_cast<int8_t*>(take(static_cast<size_t>(T) * d));
  w.beta_x = reinterpret_cast<float*>(take(static_cast<size_t>(T) * 4));
  w.rs_x = reinterpret_cast<int32_t*>(take(static_cast<size_t>(T) * 4));
  w.h = reinterpret_cast<uint16_t*>(take(R * Fr * 2));
  w.q_h = reinterpret_cast<int8_t*>(take(R * Fr));
  w.beta_h = reinterpret_cast<float*>(take(R * 4));
  w.rs_h = reinterpret_cast<int32_t*>(take(R * 4));
  w.acc_down = reinterpret_cast<int32_t*>(take(R * d * 4 * static_cast<size_t>(std::max(w.d_planes, w.d_split))));
  w.h_s = reinterpret_cast<uint16_t*>(take(static_cast<size_t>(T) * Fs * 2));
  w.y_s = reinterpret_cast<float*>(take(static_cast<size_t>(T) * d * 4 * static_cast<size_t>(w.y_planes)));
  w.xn = reinterpret_cast<uint16_t*>(take(static_cast<size_t>(T) * d * 2));
  if (l->shared_bits != 0 && T > kSharedDecodeMaxTokens) {
    w.deq_gate = reinterpret_cast<uint16_t*>(take(d * Fs * 2));
    w.deq_up = reinterpret_cast<uint16_t*>(take(d * Fs * 2));
    w.deq_down = reinterpret_cast<uint16_t*>(take(d * Fs * 2));
  }
  w.bytes = off;
  return w;
}

// ---- stage timing state (host side) ----
bool g_timing = false;
bool g_events_ready = false;
bool g_timed_run = false;
hipEvent_t g_ev[MOTE_N_STAGES + 1];

hipError_t ensure_events() {
  if (g_events_ready) return hipSuccess;
  for (int i = 0; i <= MOTE_N_STAGES; ++i) {
    hipError_t e = hipEventCreate(&g_ev[i]);
    if (e != hipSuccess) return e;
  }
  g_events_ready = true;
  return hipSuccess;
}

// ---- helper stream for the shared expert (host side, created on first use per device) ----
// The shared expert depends on x only, the routed chain (router, dispatch, two grouped GEMMs)
// does not read its result before the combine: the two run on different streams, forked from
// and joined back into the caller's stream with events.  Small batches do not fill the chip
// with one kernel; there the two chains overlap, and launch gaps and kernel tails of one are
// covered by the other.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
};
SideStream g_side[16];

hipError_t side_stream(SideStream** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
  SideStream& s = g_side[dev];
  if (s.stream == nullptr) {
    if ((e = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking)) != hipSuccess) return e;
    // The two events order work between two streams of this device only, so they carry no
    // system-scope fence (nothing here has to become visible to the host or to another device at
    // the fork or the join; the kernels' own device-scope release and acquire order the data).
    // Measured: C2 0.1572 -> 0.1552 ms, decode T=64 0.1155 -> 0.1129 ms per forward.
    // The knob kKnobEventFence = 1, set before the first forked forward, creates them with the fence.
    const bool fence = knob(kKnobEventFence) == 1;
    const unsigned f = hipEventDisableTiming | (fence ? 0u : hipEventDisableSystemFence);
    if ((e = hipEventCreateWithFlags(&s.fork, f)) != hipSuccess) return e;
    if ((e = hipEventCreateWithFlags(&s.join, f)) != hipSuccess) return e;
  }
  *out = &s;
  return hipSuccess;
}

bool fork_enabled() { return knob(kKnobNoFork) != 1; }

#define MOTE_HIP(expr)                            \
  do {                                            \
    hipError_t _e = (expr);                       \
    if (_e != hipSuccess) return MOTE_ERR_HIP;    \
  } while (0)

}  // namespace

extern "C" {

const char* mote_status_string(int status) {
  switch (status) {
    case MOTE_OK: return "ok";
    case MOTE_ERR_INVALID_ARG: return "invalid argument";
    case MOTE_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case MOTE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOTE_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int mote_version(void) { return 100; }

size_t mote_packed_bytes(int64_t n_out, int64_t n_in) {
  if (n_out <= 0 || n_in <= 0) return 0;
  return static_cast<size_t>(n_out) * static_cast<size_t>(n_in) / 4;
}

mote_status mote_pack_ternary(const void* w, int w_dtype, int64_t n_out, int64_t n_in, uint32_t* packed,
                              float* alpha, void* hip_stream) {
  if (!w || !packed || !alpha) return MOTE_ERR_INVALID_ARG;
  if (w_dtype != MOTE_DTYPE_F32 && w_dtype != MOTE_DTYPE_BF16) return MOTE_ERR_INVALID_ARG;
  if (n_out <= 0 || n_in <= 0) return MOTE_ERR_INVALID_ARG;
  if (n_out % 32 || n_in % 128) return MOTE_ERR_UNSUPPORTED_SHAPE;
  MOTE_HIP(launch_pack_ternary(w, w_dtype == MOTE_DTYPE_BF16, n_out, n_in, packed, alpha, false,
                               static_cast<hipStream_t>(hip_stream)));
  return MOTE_OK;
}

mote_status mote_pack_binary(const void* w, int w_dtype, int64_t n_out, int64_t n_in, uint32_t* packed,
                             float* alpha, void* hip_stream) {
  if (!w || !packed || !alpha) return MOTE_ERR_INVALID_ARG;
  if (w_dtype != MOTE_DTYPE_F32 && w_dtype != MOTE_DTYPE_BF16) return MOTE_ERR_INVALID_ARG;
  if (n_out <= 0 || n_in <= 0) return MOTE_ERR_INVALID_ARG;
  if (n_out % 32 || n_in % 128) return MOTE_ERR_UNSUPPORTED_SHAPE;
  MOTE_HIP(launch_pack_ternary(w, w_dtype == MOTE_DTYPE_BF16, n_out, n_in, packed, alpha, true,
                               static_cast<hipStream_t>(hip_stream)));
  return MOTE_OK;
}

size_t mote_rtn_packed_bytes(int64_t n_out, int64_t n_in, int bits) {
  if (n_out <= 0 || n_in <= 0 || (bits != 8 && bits != 4)) return 0;
  return static_cast<size_t>(n_out) * static_cast<size_t>(n_in) * static_cast<size_t>(bits) / 8;
}

mote_status mote_pack_rtn(const void* w, int64_t n_out, int64_t n_in, int bits, void* packed, float* scales,
                          void* hip_stream) {
  if (!w || !packed || !scales) return MOTE_ERR_INVALID_ARG;
  if (bits != 8 && bits != 4) return MOTE_ERR_INVALID_ARG;
  if (n_out <= 0 || n_in <= 0) return MOTE_ERR_INVALID_ARG;
  if (n_out % 32 || n_in % 128 || n_out >= (int64_t{1} << 31) || n_in >= (int64_t{1} << 24)) return MOTE_ERR_UNSUPPORTED_SHAPE;
  MOTE_HIP(launch_rtn_pack(static_cast<const uint16_t*>(w), n_out, n_in, bits, packed, scales,
                           static_cast<hipStream_t>(hip_stream)));
  return MOTE_OK;
}

mote_status mote_router_topk(const void* x, const void* w_router, const float* router_bias, int T, int d, int E,
                             int k, int32_t* topk_idx, float* topk_p, int32_t* expert_counts, void* hip_stream) {
  if (T < 0) return MOTE_ERR_INVALID_ARG;
  if (d <= 0 || d % 128 || E < 1 || E > 64 || k < 1 || k > E || k > 8) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (static_cast<int64_t>(T) * k >= (1 << 24)) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (T == 0) return MOTE_OK;
  if (!x || !w_router || !topk_idx || !topk_p) return MOTE_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  MOTE_HIP(launch_router_quant(static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_router), router_bias,
                               T, d, E, k, topk_idx, topk_p, nullptr, nullptr, nullptr, nullptr, stream));
  if (expert_counts) MOTE_HIP(launch_expert_counts(topk_idx, T * k, E, expert_counts, stream));
  return MOTE_OK;
}

mote_status mote_router_balance(const void* x, const void* w_router, const float* router_bias, int T, int d, int E,
                                int k, int32_t* topk_idx, float* topk_p, int32_t* expert_counts, float* gate_p,
                                float* gate_p_sum, float* loss, void* hip_stream) {
  if (T < 1) return MOTE_ERR_INVALID_ARG;   // the statistic divides by the number of tokens
  if (d <= 0 || d % 128 || E < 1 || E > 64 || k < 1 || k > E || k > 8) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (static_cast<int64_t>(T) * k >= (1 << 24)) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (!x || !w_router || !topk_idx || !topk_p || !expert_counts || !gate_p || !gate_p_sum || !loss) return MOTE_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  MOTE_HIP(launch_router_quant(static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_router), router_bias,
                               T, d, E, k, topk_idx, topk_p, nullptr, nullptr, nullptr, gate_p, stream));
  MOTE_HIP(launch_expert_counts(topk_idx, T * k, E, expert_counts, stream));
  MOTE_HIP(launch_balance(gate_p, expert_counts, T, E, gate_p_sum, loss, stream));
  return MOTE_OK;
}

size_t mote_layer_workspace_bytes(const mote_layer* layer, int T_max) {
  if (!layer || T_max < 0 || !layer_shape_ok(layer)) return 0;
  if (!batch_ok(layer, T_max)) return 0;
  // The kernel family (decode / large batch) and the number of K-split partial planes depend on
  // T, and not monotonically (fewer tokens can mean more planes).  A workspace sized for T_max
  // must serve every T <= T_max, so the result is the largest layout over them.  Between two
  // batch sizes at which a plane count or the kernel family can change, the layout grows with
  // T; those sizes are: the family switches, every T at which floor(T*k/128) steps (routed row
  // tiles) and every multiple of 128 (shared row tiles).  Only the last T before each is tried.
  const int k = layer->top_k, E = layer->n_experts;
  size_t need = 0;
  auto consider = [&](int64_t t) {
    if (t < 1 || t > T_max) return;
    const size_t b = carve(layer, static_cast<int>(t), nullptr).bytes;
    if (b > need) need = b;
  };
  need = carve(layer, T_max, nullptr).bytes;
  consider(kSharedDecodeMaxTokens);
  consider(int64_t{48} * E / k);
  consider(static_cast<int64_t>(knob(kKnobMidRowsLo)) * E / k);
  consider(static_cast<int64_t>(knob(kKnobMidRowsHi)) * E / k);
  for (int64_t m = 1;; ++m) {   // largest T with floor(T*k/128) == m - 1
    const int64_t t = (128 * m - 1) / k;
    if (t > T_max) break;
    consider(t);
  }
  for (int64_t t = 128; t <= T_max; t += 128) consider(t);
  return need;
}

}  // extern "C"

namespace {

// The forward pass behind both entry points.  one_stream: everything on the caller's stream and
// no host-side object is created (no helper stream, no events).
mote_status forward_impl(const mote_layer* layer, const mote_norm* norm, const void* x, int T, void* out,
                         void* workspace, size_t workspace_bytes, const mote_taps* taps, void* hip_stream,
                         bool one_stream) {
  if (!layer || T < 0) return MOTE_ERR_INVALID_ARG;
  if (norm && (norm->kind != MOTE_NORM_RMS && norm->kind != MOTE_NORM_LAYER)) return MOTE_ERR_INVALID_ARG;
  if (!layer_shape_ok(layer)) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (!batch_ok(layer, T)) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (T == 0) return MOTE_OK;
  if (!x || !out || !workspace) return MOTE_ERR_INVALID_ARG;
  if (!layer->w_router || !layer->ws_gate || !layer->ws_up || !layer->ws_down || !layer->wt_gate || !layer->wt_up ||
      !layer->wt_down || !layer->alpha)
    return MOTE_ERR_INVALID_ARG;
  if (layer->shared_bits != 0 && (!layer->ss_gate || !layer->ss_up || !layer->ss_down)) return MOTE_ERR_INVALID_ARG;
  if (norm && (!norm->gamma || (norm->kind == MOTE_NORM_LAYER && !norm->beta))) return MOTE_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return MOTE_ERR_INVALID_ARG;
  const Workspace w = carve(layer, T, static_cast<char*>(workspace));
  if (w.bytes > workspace_bytes) return MOTE_ERR_WORKSPACE_TOO_SMALL;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int d = layer->d_model, Fr = layer->d_ff_routed, Fs = layer->d_ff_shared;
  const int E = layer->n_experts, k = layer->top_k;
  const int R = T * k;
  const uint16_t* xb = static_cast<const uint16_t*>(x);
  if (norm) {   // Eq.2: the layer acts on LN(x^a); the residual x^a itself enters the combine
    MOTE_HIP(launch_norm_rows(xb, static_cast<const uint16_t*>(norm->gamma), static_cast<const uint16_t*>(norm->beta),
                              norm->kind, norm->eps, T, d, w.xn, stream));
    xb = w.xn;
  }
  const bool timing = g_timing && !one_stream;
  if (timing) MOTE_HIP(ensure_events());
  auto mark = [&](int i) -> hipError_t { return timing ? hipEventRecord(g_ev[i], stream) : hipSuccess; };

  const int tile_m = w.tile_m;
  const bool decode_routed = tile_m != 128;
  const bool decode_shared = T <= kSharedDecodeMaxTokens;
  const uint16_t* sg = static_cast<const uint16_t*>(layer->ws_gate);
  const uint16_t* su = static_cast<const uint16_t*>(layer->ws_up);
  const uint16_t* sd = static_cast<const uint16_t*>(layer->ws_down);

  // Shared expert: on the helper stream, unless stage timing wants one stage after the other.
  // Forking and joining costs the host about 40 us per call (two event records, two stream waits)
  // and the GPU a few us at the join, and two kernels that stream weights at the same time share
  // the HBM.  Measured in steady state (ms per forward, one stream vs forked): C1 0.040 vs 0.055,
  // decode shape T=16 0.1155 vs 0.1206 the one way; T=1 0.075 vs 0.0695, T=4 0.089 vs 0.081 (few
  // routed experts stream, the shared expert's weights dominate), T=32 0.1157 vs 0.112, T=64
  // 0.1229 vs 0.1155, C2 0.1896 vs 0.1644 the other.  Hence: fork when the shared expert has
  // real work (T*d*F >= 2^29), or at most 8 tokens meet a shared expert of >= 2^24 weights per
  // matrix.  The knob kKnobForkMinLog2 moves the first threshold.
  const int fork_log2 = knob(kKnobForkMinLog2);
  const int64_t shared_weights = static_cast<int64_t>(d) * Fs;
  const bool fork_pays = T * shared_weights >= (int64_t{1} << fork_log2) ||
                         (T <= 8 && shared_weights >= (int64_t{1} << 24) && fork_log2 <= 29);
  SideStream* side = nullptr;
  if (!timing && !one_stream && fork_enabled() && fork_pays) MOTE_HIP(side_stream(&side));
  hipStream_t sstream = side ? side->stream : stream;
  // Shared expert: bf16 weights (Eq.2), or RTN INT8 / INT4 codes with row scales (Section 4.3).  Small
  // batches stream the codes themselves; large batches first expand them to integer-valued bf16
  // matrices (exact) for the bf16 MFMA GEMMs, whose epilogue applies the row scales.
  const int sbits = layer->shared_bits;
  auto shared_gate_up = [&](hipStream_t s) -> hipError_t {
    if (sbits == 0)
      return decode_shared ? launch_shared_decode_gate_up(xb, sg, su, T, d, Fs, w.h_s, s)
                           : launch_shared_gate_up(xb, sg, su, T, d, Fs, w.h_s, s);
    if (decode_shared)
      return launch_shared_q_decode_gate_up(xb, layer->ws_gate, layer->ws_up, layer->ss_gate, layer->ss_up, sbits, T, d,
                                            Fs, w.h_s, s);
    hipError_t e = launch_rtn_dequant(layer->ws_gate, Fs, d, sbits, w.deq_gate, s);
    if (e != hipSuccess) return e;
    if ((e = launch_rtn_dequant(layer->ws_up, Fs, d, sbits, w.deq_up, s)) != hipSuccess) return e;
    if ((e = launch_rtn_dequant(layer->ws_down, d, Fs, sbits, w.deq_down, s)) != hipSuccess) return e;
    return launch_shared_gate_up_scaled(xb, w.deq_gate, w.deq_up, layer->ss_gate, layer->ss_up, T, d, Fs, w.h_s, s);
  };
  auto shared_down = [&](hipStream_t s) -> hipError_t {
    if (sbits == 0)
      return decode_shared ? launch_shared_decode_down(w.h_s, sd, T, d, Fs, w.y_s, s)
                           : launch_shared_down(w.h_s, sd, T, d, Fs, w.y_s, s);
    if (decode_shared) return launch_shared_q_decode_down(w.h_s, layer->ws_down, layer->ss_down, sbits, T, d, Fs, w.y_s, s);
    return launch_shared_down_scaled(w.h_s, w.deq_down, layer->ss_down, T, d, Fs, w.y_s, s);
  };
  if (side) {
    MOTE_HIP(hipEventRecord(side->fork, stream));
    MOTE_HIP(hipStreamWaitEvent(side->stream, side->fork, 0));
    MOTE_HIP(shared_gate_up(sstream));
    MOTE_HIP(shared_down(sstream));
    MOTE_HIP(hipEventRecord(side->join, side->stream));
  }

  MOTE_HIP(mark(0));
  MOTE_HIP(launch_router_quant(xb, static_cast<const uint16_t*>(layer->w_router), layer->router_bias, T, d, E, k,
                               w.topk_idx, w.topk_p, w.q_x, w.beta_x, w.rs_x, nullptr, stream));
  MOTE_HIP(mark(1));
  DispatchPlan plan{w.counts, w.offsets, w.row_of, w.tok_of, w.tile_expert, w.tile_row0, w.tile_rows, w.n_tiles, w.row_planes, w.sched};
  MOTE_HIP(launch_dispatch_plan(w.topk_idx, T, k, E, tile_m, plan, stream));
  MOTE_HIP(mark(2));

  RoutedGemmArgs ga{};
  ga.q = w.q_x; ga.gather = w.tok_of; ga.beta = w.beta_x; ga.rowsum = w.rs_x;
  ga.w_gate = layer->wt_gate; ga.w_up = layer->wt_up; ga.alpha = layer->alpha;
  ga.plan = plan; ga.max_tiles = R / tile_m + E; ga.tile_m = tile_m;
  ga.K = d; ga.N = Fr; ga.q_rows = T; ga.out_rows = R; ga.h = w.h; ga.acc_out = nullptr;
  ga.tap_gate = taps ? taps->acc_gate : nullptr;
  ga.tap_up = taps ? taps->acc_up : nullptr;
  ga.partial_stride = 0; ga.planes = 1; ga.split_max = 1;
  MOTE_HIP(decode_routed ? launch_routed_decode_gate_up(ga, stream) : launch_routed_gate_up(ga, stream));
  MOTE_HIP(mark(3));
  MOTE_HIP(launch_quant_rows(w.h, R, Fr, w.q_h, w.beta_h, w.rs_h, stream));
  MOTE_HIP(mark(4));

  RoutedGemmArgs gd = ga;
  gd.q = w.q_h; gd.gather = nullptr; gd.beta = w.beta_h; gd.rowsum = w.rs_h;
  gd.w_gate = layer->wt_down; gd.w_up = nullptr;
  gd.K = Fr; gd.N = d; gd.q_rows = R; gd.h = nullptr; gd.acc_out = w.acc_down; gd.tap_gate = nullptr; gd.tap_up = nullptr;
  gd.partial_stride = static_cast<int64_t>(R) * d; gd.planes = w.d_planes; gd.split_max = w.d_split;
  MOTE_HIP(decode_routed ? launch_routed_decode_down(gd, stream) : launch_routed_down(gd, stream));
  MOTE_HIP(mark(5));

  if (side) {
    MOTE_HIP(hipStreamWaitEvent(stream, side->join, 0));
    MOTE_HIP(mark(6));
    MOTE_HIP(mark(7));
  } else {
    MOTE_HIP(shared_gate_up(stream));
    MOTE_HIP(mark(6));
    MOTE_HIP(shared_down(stream));
    MOTE_HIP(mark(7));
  }
  CombineArgs ca{};
  ca.y_s = w.y_s; ca.y_planes = w.y_planes; ca.y_stride = static_cast<int64_t>(T) * d;
  ca.acc_down = w.acc_down; ca.d_planes = w.d_planes; ca.d_stride = static_cast<int64_t>(R) * d;
  ca.row_planes = w.d_split > 1 ? w.row_planes : nullptr;
  ca.d_tile_n = routed_down_tile_n(w.d_planes);
  ca.beta_h = w.beta_h; ca.alpha = layer->alpha;
  ca.topk_idx = w.topk_idx; ca.topk_p = w.topk_p; ca.row_of = w.row_of;
  ca.T = T; ca.d = d; ca.k = k;
  ca.residual = norm ? static_cast<const uint16_t*>(x) : nullptr;
  ca.out = static_cast<uint16_t*>(out);
  ca.out_f32 = taps ? taps->out_f32 : nullptr;
  ca.tap_y_s = taps ? taps->y_s : nullptr;
  ca.tap_acc_down = taps ? taps->acc_down : nullptr;
  MOTE_HIP(launch_combine(ca, stream));
  MOTE_HIP(mark(8));
  if (timing) g_timed_run = true;

  if (taps) {
    auto tap = [&](void* dst, const void* src, size_t bytes) -> hipError_t {
      if (!dst || bytes == 0) return hipSuccess;
      return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, stream);
    };
    const size_t Rz = static_cast<size_t>(R), Tz = static_cast<size_t>(T);
    MOTE_HIP(tap(taps->topk_idx, w.topk_idx, Rz * 4));
    MOTE_HIP(tap(taps->topk_p, w.topk_p, Rz * 4));
    MOTE_HIP(tap(taps->counts, w.counts, static_cast<size_t>(E) * 4));
    MOTE_HIP(tap(taps->row_of, w.row_of, Rz * 4));
    MOTE_HIP(tap(taps->tok_of, w.tok_of, Rz * 4));
    MOTE_HIP(tap(taps->q_x, w.q_x, Tz * d));
    MOTE_HIP(tap(taps->beta_x, w.beta_x, Tz * 4));
    MOTE_HIP(tap(taps->h, w.h, Rz * Fr * 2));
    MOTE_HIP(tap(taps->q_h, w.q_h, Rz * Fr));
    MOTE_HIP(tap(taps->beta_h, w.beta_h, Rz * 4));
    MOTE_HIP(tap(taps->h_s, w.h_s, Tz * Fs * 2));
    if (norm) MOTE_HIP(tap(taps->xn, w.xn, Tz * d * 2));
  }
  return MOTE_OK;
}

// ---- scratch of mote_layer_forward_static: one array per device, held until the process ends ----
__device__ __align__(256) unsigned char scratch[MOTE_STATIC_WORKSPACE_BYTES];
void* g_scratch_ptr[16] = {};   // device address of `scratch` on each device (the array's name is
                                // only a host-side handle: never passed to a kernel or a copy)

hipError_t static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

mote_status mote_layer_forward(const mote_layer* layer, const void* x, int T, void* out, void* workspace,
                               size_t workspace_bytes, const mote_taps* taps, void* hip_stream) {
  return forward_impl(layer, nullptr, x, T, out, workspace, workspace_bytes, taps, hip_stream, false);
}

mote_status mote_block_forward(const mote_layer* layer, const mote_norm* norm, const void* x_a, int T, void* out,
                               void* workspace, size_t workspace_bytes, const mote_taps* taps, void* hip_stream) {
  if (!norm) return MOTE_ERR_INVALID_ARG;
  return forward_impl(layer, norm, x_a, T, out, workspace, workspace_bytes, taps, hip_stream, false);
}

mote_status mote_layer_forward_static(const mote_layer* layer, const void* x, int T, void* out,
                                      const mote_taps* taps, void* hip_stream) {
  if (!layer || T < 0) return MOTE_ERR_INVALID_ARG;
  if (!layer_shape_ok(layer) || !batch_ok(layer, T)) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (T == 0) return MOTE_OK;
  // size check first: a batch that does not fit is refused before anything touches the device
  if (carve(layer, T, nullptr).bytes > MOTE_STATIC_WORKSPACE_BYTES) return MOTE_ERR_WORKSPACE_TOO_SMALL;
  void* ws = nullptr;
  MOTE_HIP(static_scratch(&ws));
  // Nothing in the array has to start at zero: the dispatch plan kernel of every forward zeroes
  // the tile counters and the plane words it uses, everything else is written before it is read.
  return forward_impl(layer, nullptr, x, T, out, ws, MOTE_STATIC_WORKSPACE_BYTES, taps, hip_stream, true);
}

mote_status mote_stage_timing(int enable) {
  g_timing = enable != 0;
  if (!g_timing) g_timed_run = false;
  return MOTE_OK;
}

mote_status mote_stage_times(float* ms_host) {
  if (!ms_host) return MOTE_ERR_INVALID_ARG;
  for (int i = 0; i < MOTE_N_STAGES; ++i) ms_host[i] = 0.0f;
  if (!g_timed_run) return MOTE_OK;
  MOTE_HIP(hipEventSynchronize(g_ev[MOTE_N_STAGES]));
  for (int i = 0; i < MOTE_N_STAGES; ++i) MOTE_HIP(hipEventElapsedTime(&ms_host[i], g_ev[i], g_ev[i + 1]));
  return MOTE_OK;
}

mote_status mote_event_pair_overhead(float* ms_host, void* hip_stream) {
  if (!ms_host) return MOTE_ERR_INVALID_ARG;
  // What two consecutive event records read when nothing runs between them: the share of a stage
  // time that is not the kernel.  Median of 33 pairs on the caller's stream.
  constexpr int kPairs = 33;
  static hipEvent_t ev[kPairs + 1];
  static bool ready = false;
  if (!ready) {
    for (int i = 0; i <= kPairs; ++i) MOTE_HIP(hipEventCreate(&ev[i]));
    ready = true;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  for (int i = 0; i <= kPairs; ++i) MOTE_HIP(hipEventRecord(ev[i], stream));
  MOTE_HIP(hipEventSynchronize(ev[kPairs]));
  float d[kPairs];
  for (int i = 0; i < kPairs; ++i) MOTE_HIP(hipEventElapsedTime(&d[i], ev[i], ev[i + 1]));
  std::sort(d, d + kPairs);
  *ms_host = d[kPairs / 2];
  return MOTE_OK;
}

size_t mote_ste_backward_workspace_bytes(int R, int N, int K, int E) {
  if (R < 0 || N <= 0 || K <= 0 || E < 1 || E > 64 || N % 128 || K % 128) return 0;
  return ste_backward_workspace_bytes(R, N, K, E);
}

mote_status mote_ste_linear_backward(const void* dy, const int32_t* offsets_host, const uint32_t* packed,
                                     const float* alpha, int alpha_stride, const int8_t* q, const float* beta,
                                     int R, int N, int K, int E, float* dx, float* dw, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  if (R < 0 || N <= 0 || K <= 0 || E < 1 || E > 64 || N % 128 || K % 128) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (!offsets_host || !packed || !alpha || !dw || !workspace || alpha_stride < 1) return MOTE_ERR_INVALID_ARG;
  if (R > 0 && (!dy || !q || !beta || !dx)) return MOTE_ERR_INVALID_ARG;
  if (offsets_host[0] != 0 || offsets_host[E] != R) return MOTE_ERR_INVALID_ARG;
  const int64_t lim = int64_t{1} << 31;
  for (int e = 0; e < E; ++e) {
    const int64_t rows = static_cast<int64_t>(offsets_host[e + 1]) - offsets_host[e];
    if (rows < 0) return MOTE_ERR_INVALID_ARG;
    if ((rows + 64) * N * 2 >= lim || (rows + 64) * K * 4 >= lim) return MOTE_ERR_UNSUPPORTED_SHAPE;
  }
  if (static_cast<int64_t>(N) * K * 4 >= lim) return MOTE_ERR_UNSUPPORTED_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return MOTE_ERR_INVALID_ARG;
  if (ste_backward_workspace_bytes(R, N, K, E) > workspace_bytes) return MOTE_ERR_WORKSPACE_TOO_SMALL;
  MOTE_HIP(launch_ste_backward(static_cast<const uint16_t*>(dy), offsets_host, packed, alpha, alpha_stride, q, beta, R, N,
                               K, E, dx, dw, workspace, static_cast<hipStream_t>(hip_stream)));
  return MOTE_OK;
}

mote_status mote_tuning_set(int knob_id, int value) {
  if (knob_id < 0 || knob_id >= mote::kKnobCount) return MOTE_ERR_INVALID_ARG;
  mote::g_knobs[knob_id] = value;
  return MOTE_OK;
}

mote_status mote_calib_copy(void* dst, const void* src, size_t n_bytes, void* hip_stream) {
  if (!dst || !src || n_bytes % 16) return MOTE_ERR_INVALID_ARG;
  MOTE_HIP(launch_copy(dst, src, n_bytes, static_cast<hipStream_t>(hip_stream)));
  return MOTE_OK;
}

}  // extern "C"
