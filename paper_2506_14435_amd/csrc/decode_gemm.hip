// Small-batch (decode) GEMMs of the MoTE layer: the weights are streamed from HBM exactly
// once and every design choice serves bytes in flight, not MFMA rate.
//
//   routed_wave_kernel<0/1>:   ternary gate-up (Eq.6) / down (Eq.5) when there are enough (row tile,
//                              fragment) units for every wavefront of the chip: activation plane in
//                              LDS, each wavefront streams whole fragments through a register ring
//   routed_stream_kernel<0/1>: the same for fewer rows: the four wavefronts of a workgroup split K
//   routed_decode_kernel<0/1>: register-ring fallback for d_model > 2048 (gate-up planes longer
//                              than 16 K steps)
//   shared_wave_kernel<0/1>:   bf16 shared expert (Eq.2) for T <= 64 tokens, one wavefront per
//                              workgroup with a private LDS ring
//
// Cross-workgroup K splits (down projections) are written as separate partial planes that the
// combine kernel adds in a fixed order, so the result does not depend on scheduling.
//
// MFMA operand mapping as in the large-batch kernels: first operand = weights (lane l:
// output channel l%32, K half l/32), second = activations (lane l: row l%32); result
// register v of lane l is output channel 8*(v/4) + 4*(l/32) + v%4 of row l%32.
//
// routed_decode_kernel: a workgroup of four wavefronts owns one 32-channel fragment of the output
// (both matrices in gate-up mode) and splits the contraction length four ways.  A wavefront keeps
// a ring of PD K steps in registers: the weight loads (one 16-byte load per lane = 1 KiB per
// packed ternary tile) and the matching activation fragments are issued PD steps ahead of the
// MFMAs that consume them, nothing is staged in LDS and there is no barrier in the K loop.  The
// four partial accumulators meet in LDS, where the epilogue of the large-batch kernels is applied.
#include <stdlib.h>

#include <algorithm>
#include "common.h"
#include "launch.h"

namespace mote {

constexpr int kDecThreads = 256;

// ------------------------------------------------------------------------- routed experts
template <int MODE>
__global__ __launch_bounds__(kDecThreads) void routed_decode_kernel(RoutedGemmArgs a, int n_frags, int kc_count,
                                                                    int steps_per_wave) {
  constexpr int NMAT = MODE == 0 ? 2 : 1;
  constexpr int PD = 4;
  __shared__ int s_part[4 * NMAT * 16 * 64];

  const int K = a.K, N = a.N, KT = K >> 7;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, g = lane >> 5;
  const int64_t expert_bytes = static_cast<int64_t>(N) * K / 4;
  const int n_tiles = a.plan.n_tiles[0];
  const int units = n_tiles * n_frags * kc_count;

  for (int u = blockIdx.x; u < units; u += gridDim.x) {
    const int kc = u % kc_count;
    const int nf = (u / kc_count) % n_frags;
    const int mt = u / (kc_count * n_frags);
    const int expert = a.plan.tile_expert[mt];
    const int row0 = a.plan.tile_row0[mt];
    const int rows = a.plan.tile_rows[mt];
    const int step0 = (kc * 4 + wave) * steps_per_wave;
    const int nsteps = max(0, min(steps_per_wave, KT - step0));

    // weight ring first: it does not depend on the row gather
    const unsigned char* wg = reinterpret_cast<const unsigned char*>(a.w_gate) + expert * expert_bytes +
                              (static_cast<int64_t>(nf) * KT + step0) * 1024 + lane * 16;
    const unsigned char* wu = nullptr;
    if constexpr (NMAT == 2)
      wu = reinterpret_cast<const unsigned char*>(a.w_up) + expert * expert_bytes +
           (static_cast<int64_t>(nf) * KT + step0) * 1024 + lane * 16;
    u4 wr[PD][NMAT];
    v4i ar[PD][4];
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      if (j < nsteps) {
        wr[j][0] = __builtin_nontemporal_load(reinterpret_cast<const u4*>(wg + j * 1024));
        if constexpr (NMAT == 2) wr[j][1] = __builtin_nontemporal_load(reinterpret_cast<const u4*>(wu + j * 1024));
      }
    }
    // activation rows: lane (r32, g) reads 16 bytes per 32-channel sub-step
    const int slot = row0 + min(r32, rows - 1);
    const int src = a.gather ? a.gather[slot] : slot;
    const unsigned char* ap = reinterpret_cast<const unsigned char*>(a.q) + static_cast<int64_t>(src) * K +
                              static_cast<int64_t>(step0) * 128 + g * 16;
    // epilogue metadata of the row this thread finishes (row tid % 32)
    const float m_beta = a.beta[src];
    const int m_rs = a.rowsum[src];
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      if (j < nsteps) {
#pragma unroll
        for (int s = 0; s < 4; ++s) ar[j][s] = *reinterpret_cast<const v4i*>(ap + j * 128 + s * 32);
      }
    }

    v16i acc[NMAT];
#pragma unroll
    for (int m = 0; m < NMAT; ++m)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[m][v] = 0;

    for (int base = 0; base < nsteps; base += PD) {
#pragma unroll
      for (int j = 0; j < PD; ++j) {
        if (base + j < nsteps) {
#pragma unroll
          for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int m = 0; m < NMAT; ++m)
              acc[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(unpack_codes(wr[j][m][s]), ar[j][s], acc[m], 0, 0, 0);
          }
          const int nx = base + j + PD;
          if (nx < nsteps) {
            wr[j][0] = __builtin_nontemporal_load(reinterpret_cast<const u4*>(wg + static_cast<int64_t>(nx) * 1024));
            if constexpr (NMAT == 2) wr[j][1] = __builtin_nontemporal_load(reinterpret_cast<const u4*>(wu + static_cast<int64_t>(nx) * 1024));
#pragma unroll
            for (int s = 0; s < 4; ++s)
              ar[j][s] = *reinterpret_cast<const v4i*>(ap + static_cast<int64_t>(nx) * 128 + s * 32);
          }
        }
      }
    }

    // partial accumulators of the four K slices meet in LDS
#pragma unroll
    for (int m = 0; m < NMAT; ++m)
#pragma unroll
      for (int v = 0; v < 16; ++v) s_part[((wave * NMAT + m) * 16 + v) * 64 + lane] = acc[m][v];
    __syncthreads();
    // thread t finishes register quad q = t / 64 of lane t % 64: row (t % 32), four channels
    {
      const int q = tid >> 6;
      int sum[NMAT][4];
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          int t = 0;
#pragma unroll
          for (int w = 0; w < 4; ++w) t += s_part[((w * NMAT + m) * 16 + 4 * q + j) * 64 + lane];
          sum[m][j] = t;
        }
      if (r32 < rows) {
        const int n = nf * 32 + 8 * q + 4 * g;
        const int64_t o = static_cast<int64_t>(row0 + r32) * N + n;
        if constexpr (MODE == 0) {
          const float sx = m_beta / 127.0f;
          const float sg = sx * a.alpha[expert * 3 + 0], su = sx * a.alpha[expert * 3 + 1];
          float hv[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            sum[0][j] -= m_rs;
            sum[1][j] -= m_rs;
            hv[j] = (static_cast<float>(sum[1][j]) * su) * silu_fast(static_cast<float>(sum[0][j]) * sg);
          }
          uint2 packed;
          packed.x = cvt_pk_bf16(hv[0], hv[1]);
          packed.y = cvt_pk_bf16(hv[2], hv[3]);
          *reinterpret_cast<uint2*>(a.h + o) = packed;
          if (a.tap_gate != nullptr)
            *reinterpret_cast<int4*>(a.tap_gate + o) = make_int4(sum[0][0], sum[0][1], sum[0][2], sum[0][3]);
          if (a.tap_up != nullptr)
            *reinterpret_cast<int4*>(a.tap_up + o) = make_int4(sum[1][0], sum[1][1], sum[1][2], sum[1][3]);
        } else {
          const int corr = kc == 0 ? m_rs : 0;   // the zero-point correction enters exactly one partial plane
          *reinterpret_cast<int4*>(a.acc_out + static_cast<int64_t>(kc) * a.partial_stride + o) =
              make_int4(sum[0][0] - corr, sum[0][1] - corr, sum[0][2] - corr, sum[0][3] - corr);
        }
      }
    }
    __syncthreads();
  }
}

// Streaming variant: a workgroup owns a contiguous run of output fragments of one
// (row tile, K plane).  Each wavefront keeps its activation fragments for its four K steps
// resident in registers for the whole run and streams only packed weights, two fragments
// ahead (register double buffer refilled the moment a fragment has been consumed), so the
// weight loads stay in flight across the per-fragment reduction and epilogue.  The LDS
// reduction buffer is double buffered: one barrier per fragment.
// Requires K <= 2048 per plane: gate-up with d_model <= 2048, and every down plane.
template <int MODE>
__global__ __launch_bounds__(kDecThreads, 2) void routed_stream_kernel(RoutedGemmArgs a, int n_frags, int kc_count) {
  constexpr int NMAT = MODE == 0 ? 2 : 1;
  __shared__ __attribute__((aligned(16))) int s_part[2][4 * NMAT * 16 * 64];

  const int K = a.K, N = a.N, KT = K >> 7;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, g = lane >> 5, q = tid >> 6;
  const int64_t expert_bytes = static_cast<int64_t>(N) * K / 4;
  const int64_t frag_bytes = static_cast<int64_t>(KT) * 1024;
  const int64_t total = static_cast<int64_t>(a.plan.n_tiles[0]) * kc_count * n_frags;
  int64_t u = blockIdx.x * total / gridDim.x;
  const int64_t hi = (blockIdx.x + 1) * total / gridDim.x;
  int buf = 0;

  while (u < hi) {
    const int grp = static_cast<int>(u / n_frags);          // (row tile, K plane)
    const int nf0 = static_cast<int>(u - static_cast<int64_t>(grp) * n_frags);
    const int nf_end = static_cast<int>(min(static_cast<int64_t>(n_frags), nf0 + (hi - u)));
    const int mt = grp / kc_count, kc = grp - mt * kc_count;
    const int expert = a.plan.tile_expert[mt];
    const int row0 = a.plan.tile_row0[mt];
    const int rows = a.plan.tile_rows[mt];
    const int step0 = (kc * 4 + wave) * 4;
    const int nsteps = max(0, min(4, KT - step0));

    const unsigned char* wb[NMAT];
    wb[0] = reinterpret_cast<const unsigned char*>(a.w_gate) + expert * expert_bytes +
            static_cast<int64_t>(step0) * 1024 + lane * 16;
    if constexpr (NMAT == 2)
      wb[1] = reinterpret_cast<const unsigned char*>(a.w_up) + expert * expert_bytes +
              static_cast<int64_t>(step0) * 1024 + lane * 16;
    u4 w_a[NMAT][4], w_b[NMAT][4];
#define MOTE_LOADW(dst_, nf_)                                                               \
  _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                          \
    _Pragma("unroll") for (int s = 0; s < 4; ++s)                                           \
      if (s < nsteps) dst_[m][s] = __builtin_nontemporal_load(reinterpret_cast<const u4*>(wb[m] + (nf_) * frag_bytes + s * 1024))
    MOTE_LOADW(w_a, nf0);
    if (nf0 + 1 < nf_end) { MOTE_LOADW(w_b, nf0 + 1); }

    // resident activation fragments of this wavefront's K slice
    const int slot = row0 + min(r32, rows - 1);
    const int src = a.gather ? a.gather[slot] : slot;
    const unsigned char* ap = reinterpret_cast<const unsigned char*>(a.q) + static_cast<int64_t>(src) * K +
                              static_cast<int64_t>(step0) * 128 + g * 16;
    const float m_beta = a.beta[src];
    const int m_rs = a.rowsum[src];
    v4i ar[4][4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
      if (s < nsteps) {
#pragma unroll
        for (int b = 0; b < 4; ++b) ar[s][b] = *reinterpret_cast<const v4i*>(ap + s * 128 + b * 32);
      }
    float sg = 0.0f, su = 0.0f;
    if constexpr (MODE == 0) {
      const float sx = m_beta / 127.0f;
      sg = sx * a.alpha[expert * 3 + 0];
      su = sx * a.alpha[expert * 3 + 1];
    }
    const int corr = (MODE == 0 || kc == 0) ? m_rs : 0;   // zero-point correction enters one plane only

#define MOTE_FRAG(w_, nf_, nxt_)                                                                          \
  {                                                                                                       \
    v16i acc[NMAT];                                                                                       \
    _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                                      \
      _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[m][v] = 0;                                       \
    _Pragma("unroll") for (int s = 0; s < 4; ++s)                                                         \
      if (s < nsteps) {                                                                                   \
        _Pragma("unroll") for (int b = 0; b < 4; ++b)                                                     \
          _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                                \
            acc[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(unpack_codes(w_[m][s][b]), ar[s][b],       \
                                                           acc[m], 0, 0, 0);                              \
      }                                                                                                   \
    if ((nxt_) < nf_end) { MOTE_LOADW(w_, (nxt_)); }                                                      \
    v4i* part = reinterpret_cast<v4i*>(s_part[buf]);   /* [wave][matrix][quad][lane] of 4 ints */         \
    _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                                      \
      _Pragma("unroll") for (int qq = 0; qq < 4; ++qq) {                                                  \
        v4i t4 = {acc[m][4 * qq], acc[m][4 * qq + 1], acc[m][4 * qq + 2], acc[m][4 * qq + 3]};            \
        part[((wave * NMAT + m) * 4 + qq) * 64 + lane] = t4;                                              \
      }                                                                                                   \
    __syncthreads();                                                                                      \
    int sum[NMAT][4];                                                                                     \
    _Pragma("unroll") for (int m = 0; m < NMAT; ++m) {                                                    \
      v4i t4 = {-corr, -corr, -corr, -corr};                                                              \
      _Pragma("unroll") for (int w = 0; w < 4; ++w) t4 += part[((w * NMAT + m) * 4 + q) * 64 + lane];     \
      sum[m][0] = t4.x; sum[m][1] = t4.y; sum[m][2] = t4.z; sum[m][3] = t4.w;                             \
    }                                                                                                     \
    buf ^= 1;                                                                                             \
    if (r32 < rows) {                                                                                     \
      const int64_t o = static_cast<int64_t>(row0 + r32) * N + (nf_) * 32 + 8 * q + 4 * g;               \
      if constexpr (MODE == 0) {                                                                          \
        float hv[4];                                                                                      \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                     \
          hv[j] = (static_cast<float>(sum[NMAT - 1][j]) * su) * silu_fast(static_cast<float>(sum[0][j]) * sg); \
        uint2 packed;                                                                                     \
        packed.x = cvt_pk_bf16(hv[0], hv[1]);                                                             \
        packed.y = cvt_pk_bf16(hv[2], hv[3]);                                                             \
        *reinterpret_cast<uint2*>(a.h + o) = packed;                                                      \
        if (a.tap_gate != nullptr)                                                                        \
          *reinterpret_cast<int4*>(a.tap_gate + o) = make_int4(sum[0][0], sum[0][1], sum[0][2], sum[0][3]); \
        if (a.tap_up != nullptr)                                                                          \
          *reinterpret_cast<int4*>(a.tap_up + o) =                                                        \
              make_int4(sum[NMAT - 1][0], sum[NMAT - 1][1], sum[NMAT - 1][2], sum[NMAT - 1][3]);          \
      } else {                                                                                            \
        *reinterpret_cast<int4*>(a.acc_out + static_cast<int64_t>(kc) * a.partial_stride + o) =           \
            make_int4(sum[0][0], sum[0][1], sum[0][2], sum[0][3]);                                        \
      }                                                                                                   \
    }                                                                                                     \
  }
    for (int nf = nf0; nf < nf_end; nf += 2) {
      MOTE_FRAG(w_a, nf, nf + 2);
      if (nf + 1 < nf_end) MOTE_FRAG(w_b, nf + 1, nf + 3);
    }
#undef MOTE_FRAG
#undef MOTE_LOADW
    u += nf_end - nf0;
  }
}

// Wave-streaming variant for many (tile, fragment) units: the int8 activation rows of one
// (row tile, K plane of 16 steps) sit in LDS (64 KiB, loaded directly from global memory),
// and every wavefront of the workgroup owns whole output fragments of that tile: it streams the
// packed weights of its fragment through a register ring of eight K steps, crossing into its
// next fragment without a bubble, and finishes the fragment alone - no barrier, no cross-wave
// reduction in the steady state.  Loads are raw buffer loads issued unconditionally (a lane
// offset beyond the buffer turns one into a no-op), so the number of loads in flight is the
// same on every path and the compiler's wait counts stay exact.  A plane shorter than 16 steps
// is padded with zero activations (the weights of the padding are not fetched).
// The grid is two workgroups per CU; each (row tile, K plane) group is shared evenly by
// floor(grid / groups) workgroups, so a workgroup stays with one plane (changing it cost a drained
// load queue and two barriers) and every CU streams about the same number of bytes.  That
// balance matters more than an equal number of fragments per wavefront: a CU serves its own
// requests in order at its share of the HBM bandwidth, and with 352 equal workgroups on 256 CUs
// the CUs that held two finished at 37 us, the others at 23 us (measured).
// The plane is requested before the first weights: vector-memory operations complete in issue
// order, so "all but the ring's loads" retires the plane while the weights keep streaming.
#ifdef MOTE_TRACE_DEC
__device__ unsigned long long g_dtrace[1024 * 4 * 24];
#define MOTE_DTP(k_) if (MODE == MOTE_TRACE_DEC && lane == 0 && (k_) < 24) g_dtrace[(blockIdx.x * NW + wave) * 24 + (k_)] = wall_clock64();
extern "C" int mote_debug_dtrace(void* dst, size_t bytes) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_dtrace), bytes); }
#else
#define MOTE_DTP(k_)
#endif

// MF: 32-row fragments of a row tile (plan tiles of 32 * MF rows), NW: wavefronts of the workgroup,
// which share one plane: 64 KiB (MF = 1) or 128 KiB (MF = 2: experts with some tens of rows each;
// every unpacked weight fragment feeds two MFMAs).  Eight wavefronts in one workgroup per CU beat
// two workgroups of four: the second workgroup of a CU got its plane 4-5 us after the first (its
// loads queue behind the first one's weight ring) and ended 6 us later; alone the kernel takes the
// same time either way, beside the shared expert's kernels the forward is 3-7 % faster (T = 16..64).
template <int MODE, int MF, int NW>
__global__ __launch_bounds__(64 * NW, 2) void routed_wave_kernel(RoutedGemmArgs a, int n_frags, int kc_count) {
  constexpr int NMAT = MODE == 0 ? 2 : 1;
  constexpr int NT = 64 * NW;                             // threads of the workgroup (NW wavefronts)
  constexpr int RB = 4 * MF;                              // blocks of eight rows in the plane
  static_assert(NW % RB == 0, "a wavefront loads one row block of the plane");
  constexpr int ROWS = 32 * MF;                           // rows of the plane
  constexpr int STEP_BYTES = ROWS * 128;                  // one K step of the plane
  constexpr int D = 8;                                    // K steps of packed weights in flight per wavefront (16 measured no faster)
  constexpr int DF = 4;                                   // ... of which this many are requested before the plane
  constexpr int kBufferFlags = 0x00020000;                // raw buffer, 32-bit data format
  constexpr int kWeightAux = 2;                           // weight loads are non-temporal: every byte is used once (measured: 42 -> 39.5 us)
  constexpr uint32_t kOutOfRange = 0x80000000u;           // lane offset past any buffer of <= 2 GiB
  // activations of the plane: [K step 16][block of 8 rows][position 8][row of the block 8][16 bytes],
  // the 16-byte chunk c of a row sits at position c ^ (block & 1): a quarter wavefront reads one chunk
  // of 16 consecutive rows = two runs of 128 bytes in different halves of the 64 banks
  extern __shared__ __attribute__((aligned(16))) unsigned char s_a[];

  const int K = a.K, N = a.N, KT = K >> 7;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, g = lane >> 5;
  const int64_t expert_words = static_cast<int64_t>(N) * K / 16;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)s_a);
  // MFMA operand of lane (r32, g), fragment f, sub-step s of K step kt: chunk 2s + g of row 32f + r32
  const int a_lane = (r32 >> 3) * 1024 + (((g ^ ((r32 >> 3) & 1)) * 8 + (r32 & 7)) << 4);
  auto make_rsrc = [&](const void* base, int64_t bytes) {
    const uint64_t p = reinterpret_cast<uint64_t>(base);
    v4i r;
    r.x = static_cast<int>(static_cast<uint32_t>(p));
    r.y = static_cast<int>(static_cast<uint32_t>(p >> 32) & 0xFFFFu);
    r.z = static_cast<int>(bytes);
    r.w = kBufferFlags;
    return r;
  };
  const v4i rsrc_q = make_rsrc(a.q, a.q_rows * K);
  // The tile list (at most 64 entries here) is fetched whole, lane l entry l, beside the tile
  // count it depends on: the weights can then be requested after one memory round trip.
  const bool tile_table = a.max_tiles <= 64;
  int t_expert = 0, t_row0 = 0, t_rows = 0;
  if (tile_table && lane < a.max_tiles) {
    t_expert = a.plan.tile_expert[lane];
    t_row0 = a.plan.tile_row0[lane];
    t_rows = a.plan.tile_rows[lane];
  }
  const int groups = load_uniform(a.plan.n_tiles) * kc_count;
  // Each (row tile, K plane) group is shared evenly by floor(grid / groups) workgroups.  Where that
  // would leave more than a quarter of the grid idle (MF = 2: one workgroup per CU, groups often
  // between half the grid and the grid), the (group, fragment) units are cut into equal runs instead
  // and a workgroup may end one group and start the next (slower per unit: two plane loads).
  const int bpg = max(1, static_cast<int>(gridDim.x) / max(groups, 1));   // workgroups per (row tile, K plane) group
  const int gstride = gridDim.x / bpg;                                     // groups in flight
  const int g0 = blockIdx.x / bpg, part = blockIdx.x - g0 * bpg;
  const bool even = MF == 2 && static_cast<int64_t>(bpg) * min(groups, gstride) * 4 < static_cast<int64_t>(gridDim.x) * 3;
  if (!even && g0 >= gstride) return;                                      // left-over workgroups
  const int64_t units = static_cast<int64_t>(groups) * n_frags;
  int64_t u = static_cast<int64_t>(blockIdx.x) * units / gridDim.x;
  const int64_t u_end = static_cast<int64_t>(blockIdx.x + 1) * units / gridDim.x;
  int tp = 0;
  MOTE_DTP(tp) ++tp;
  bool first = true;
  for (int grp = even ? static_cast<int>(u / n_frags) : g0; even ? u < u_end : grp < groups;) {
    // every wavefront is done with the previous plane (a plain barrier: the loads in flight stay in flight)
    if (!first) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    first = false;
    int nf0, nf_end;
    if (!even) {
      nf0 = part * n_frags / bpg;
      nf_end = (part + 1) * n_frags / bpg;
    } else {
      nf0 = static_cast<int>(u - static_cast<int64_t>(grp) * n_frags);
      nf_end = static_cast<int>(min(static_cast<int64_t>(n_frags), nf0 + (u_end - u)));
    }
    const int mt = grp / kc_count, kc = grp - mt * kc_count;
    const int expert = tile_table ? __builtin_amdgcn_readlane(t_expert, mt) : load_uniform(a.plan.tile_expert + mt);
    const int row0 = tile_table ? __builtin_amdgcn_readlane(t_row0, mt) : load_uniform(a.plan.tile_row0 + mt);
    const int rows = tile_table ? __builtin_amdgcn_readlane(t_rows, mt) : load_uniform(a.plan.tile_rows + mt);
    // the K planes share the contraction evenly (at most 16 steps each): with planes of 16 steps and
    // a short last one, the workgroups of the last plane had a third of the bytes of the others
    const int step0 = kc * KT / kc_count;
    const int nsteps = (kc + 1) * KT / kc_count - step0;

    // Order of the requests (vector-memory operations complete in issue order): the row indices
    // the plane depends on, the first half of the weight ring (it needs only the tile's expert:
    // HBM is busy from here on), the row scales, the plane, the rest of the ring.
    // Plane: a load fills 1 KiB with the 128 bytes of a K step of eight rows (lane l: row l % 8
    // of the block, position l / 8): whole cache lines.  Wavefront w loads row block w % RB of
    // every (NW / RB)-th K step.  Rows past the end of the tile are not fetched (their accumulator
    // rows are never stored).
    const int lblock = wave % RB;
    const int lrow = lblock * 8 + (lane & 7);
    const int lslot = row0 + min(lrow, rows - 1);
    const int lsrc = a.gather ? a.gather[lslot] : lslot;
    int src_f[MF];   // rows of this lane in the MFMA layout: fragment f holds row 32 f + r32
#pragma unroll
    for (int f = 0; f < MF; ++f) {
      const int slot = row0 + min(f * 32 + r32, rows - 1);
      src_f[f] = a.gather ? a.gather[slot] : slot;
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- weight ring, first half ----
    __amdgpu_buffer_rsrc_t rw[NMAT];
    rw[0] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.w_gate) + expert * expert_words, 0,
                                              static_cast<int>(expert_words * 4), kBufferFlags);
    if constexpr (NMAT == 2)
      rw[1] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.w_up) + expert * expert_words, 0,
                                                static_cast<int>(expert_words * 4), kBufferFlags);
    const uint32_t w_lane = lane * 16;
    u4 wr[D][NMAT];
    int nf = nf0 + wave;   // this wavefront's fragments: nf0 + wave, + NW, ...
    const uint32_t oob = nf < nf_end ? 0u : kOutOfRange;   // out of range if this wavefront has no fragment
#pragma unroll
    for (int j = 0; j < DF; ++j)
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
        wr[j][m] = __builtin_amdgcn_raw_buffer_load_b128(rw[m], w_lane + (j < nsteps ? oob : kOutOfRange),
                                                         (nf * KT + step0 + j) * 1024, kWeightAux);
    __builtin_amdgcn_sched_barrier(0);

    // the row scales before the plane: the compiler does not see the plane's loads, and its wait for
    // the row indices would otherwise count them as the first half of the ring
    float m_beta[MF];
    int m_rs[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f) {
      m_beta[f] = a.beta[src_f[f]];
      m_rs[f] = a.rowsum[src_f[f]];
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- activation plane into LDS ----
    {
      const uint32_t voff = lrow < rows ? static_cast<uint32_t>(lsrc) * static_cast<uint32_t>(K) + step0 * 128 +
                                              (((lane >> 3) ^ (lblock & 1)) << 4)
                                        : kOutOfRange;
      for (int st = wave / RB; st < nsteps; st += NW / RB) {
        const uint32_t dst = lds0 + static_cast<uint32_t>(st * STEP_BYTES + lblock * 1024);
        const int soff = st * 128;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :: "s"(dst), "v"(voff), "s"(rsrc_q), "s"(soff) : "memory");
      }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- weight ring, second half ----
#pragma unroll
    for (int j = DF; j < D; ++j)
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
        wr[j][m] = __builtin_amdgcn_raw_buffer_load_b128(rw[m], w_lane + (j < nsteps ? oob : kOutOfRange),
                                                         (nf * KT + step0 + j) * 1024, kWeightAux);
    __builtin_amdgcn_sched_barrier(0);

    // steps past the end of the contraction contribute nothing: zero activations
    for (int i = nsteps * 256 * MF + tid; i < 16 * 256 * MF; i += NT)   // 256 * MF x 16 bytes per K step
      *reinterpret_cast<u4*>(s_a + i * 16) = u4{0u, 0u, 0u, 0u};
    float sg[MF], su[MF];
    int corr[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f) {
      sg[f] = 0.0f; su[f] = 0.0f;
      if constexpr (MODE == 0) {
        const float sx = m_beta[f] / 127.0f;
        sg[f] = sx * load_uniform(a.alpha + expert * 3 + 0);
        su[f] = sx * load_uniform(a.alpha + expert * 3 + 1);
      }
      corr[f] = (MODE == 0 || kc == 0) ? m_rs[f] : 0;   // zero-point correction enters one plane only
    }
    const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(
        MODE == 0 ? static_cast<void*>(a.h) : static_cast<void*>(a.acc_out + static_cast<int64_t>(kc) * a.partial_stride), 0,
        static_cast<int>(a.out_rows * N * (MODE == 0 ? 2 : 4)), kBufferFlags);
    MOTE_DTP(tp) ++tp;
    // the plane and the row metadata (everything requested before the second half of the ring) have landed;
    // that half stays in flight (a plain barrier: __syncthreads() would also drain it)
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"((D - DF) * NMAT) : "memory");
    MOTE_DTP(tp) ++tp;

    for (; nf < nf_end; nf += NW) {
      const uint32_t oob_next = nf + NW < nf_end ? 0u : kOutOfRange;
      v16i acc[NMAT][MF];
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < MF; ++f)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[m][f][v] = 0;
#pragma unroll
      for (int kt = 0; kt < 16; ++kt) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          v4i af[MF];
#pragma unroll
          for (int f = 0; f < MF; ++f)
            af[f] = *reinterpret_cast<const v4i*>(s_a + kt * STEP_BYTES + f * 4096 + s * 256 + a_lane);
#pragma unroll
          for (int m = 0; m < NMAT; ++m) {
            const v4i wf = unpack_codes(wr[kt % D][m][s]);
#pragma unroll
            for (int f = 0; f < MF; ++f)
              acc[m][f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, af[f], acc[m][f], 0, 0, 0);
          }
        }
        // refill the slot: step kt + D of this fragment, or step kt + D - 16 of the next one
#pragma unroll
        for (int m = 0; m < NMAT; ++m) {
          // steps of the padding are not fetched (a lane offset out of range: no traffic, zeros back)
          if (kt + D < 16)
            wr[kt % D][m] = __builtin_amdgcn_raw_buffer_load_b128(rw[m], w_lane + (kt + D < nsteps ? 0u : kOutOfRange),
                                                                  (nf * KT + step0 + kt + D) * 1024, kWeightAux);
          else
            wr[kt % D][m] = __builtin_amdgcn_raw_buffer_load_b128(rw[m], w_lane + (kt + D - 16 < nsteps ? oob_next : kOutOfRange),
                                                                  ((nf + NW) * KT + step0 + kt + D - 16) * 1024, kWeightAux);
        }
        __builtin_amdgcn_sched_barrier(0);   // one K step at a time: the LDS reads of later steps would pile up in registers
      }
      // ---- epilogue of the fragment: lane l owns rows 32 f + r32 and channels 8q + 4g .. +3 ----
#pragma unroll
      for (int f = 0; f < MF; ++f) {
        const bool row_ok = f * 32 + r32 < rows;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint32_t o = static_cast<uint32_t>(row0 + f * 32 + r32) * static_cast<uint32_t>(N) + nf * 32 + 8 * q + 4 * g;
          int sum[NMAT][4];
#pragma unroll
          for (int m = 0; m < NMAT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) sum[m][j] = acc[m][f][4 * q + j] - corr[f];
          if constexpr (MODE == 0) {
            float hv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
              hv[j] = (static_cast<float>(sum[NMAT - 1][j]) * su[f]) * silu_fast(static_cast<float>(sum[0][j]) * sg[f]);
            typedef unsigned u2v __attribute__((ext_vector_type(2)));
            u2v packed;
            packed.x = cvt_pk_bf16(hv[0], hv[1]);
            packed.y = cvt_pk_bf16(hv[2], hv[3]);
            __builtin_amdgcn_raw_buffer_store_b64(packed, r_out, row_ok ? o * 2u : kOutOfRange, 0, 0);
            if (row_ok && a.tap_gate != nullptr)
              *reinterpret_cast<int4*>(a.tap_gate + o) = make_int4(sum[0][0], sum[0][1], sum[0][2], sum[0][3]);
            if (row_ok && a.tap_up != nullptr)
              *reinterpret_cast<int4*>(a.tap_up + o) =
                  make_int4(sum[NMAT - 1][0], sum[NMAT - 1][1], sum[NMAT - 1][2], sum[NMAT - 1][3]);
          } else {
            const u4 d4 = {static_cast<unsigned>(sum[0][0]), static_cast<unsigned>(sum[0][1]),
                           static_cast<unsigned>(sum[0][2]), static_cast<unsigned>(sum[0][3])};
            __builtin_amdgcn_raw_buffer_store_b128(d4, r_out, row_ok ? o * 4u : kOutOfRange, 0, 0);
          }
        }
      }
      MOTE_DTP(tp) ++tp;
    }
    if (!even) {
      grp += gstride;
    } else {
      u += nf_end - nf0;
      ++grp;
    }
  }
  MOTE_DTP(tp) ++tp;
  MOTE_DTP(23)
}

static int device_cus() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
  }
  return n;
}

int routed_decode_down_planes(int K) { return ((K >> 7) + 15) / 16; }

template <int MODE, int MF, int NW>
static hipError_t launch_wave(const RoutedGemmArgs& a, int n_frags, int kc, hipStream_t stream) {
  constexpr int kLds = 16 * 8 * 32 * MF * 16;   // the activation plane
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(routed_wave_kernel<MODE, MF, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  routed_wave_kernel<MODE, MF, NW><<<device_cus() * (8 / NW), 64 * NW, kLds, stream>>>(a, n_frags, kc);
  return hipGetLastError();
}

// Plan tiles of 64 rows (experts with some tens of rows each) always run the wave-streaming kernel:
// the shape must give it whole planes and enough fragments.
bool routed_mid_kernel_fits(int d, int F) {
  const int KTg = d >> 7, KTd = F >> 7;
  if (KTg > 16 || 16 * 3 > KTg * 4) return false;                        // gate-up: one plane, at most a third of it padding
  const int kc = routed_decode_down_planes(F);
  if (kc * 16 * 3 > KTd * 4) return false;
  return F / 32 >= 256 && static_cast<int64_t>(d / 32) * kc >= 192;
}

// The wave-streaming kernel wants whole 16-step planes (a ragged last plane is padded with
// zero activations) and enough units to give every wavefront of the grid a fragment.
static bool use_wave_kernel(const RoutedGemmArgs& a, int n_frags, int kc) {
  const int forced = knob(kKnobDecodeVariant);
  if (forced >= 0) return forced >= 1;
  const int KT = a.K >> 7;
  const int padded = kc * 16;
  if (padded * 3 > KT * 4) return false;                                 // more than a third of the MFMA work would be padding
  if (static_cast<int64_t>(a.q_rows) * a.K >= (int64_t{1} << 31)) return false;
  // few dispatch rows = few row tiles: the K-split kernel keeps all four wavefronts of a workgroup busy then
  return a.out_rows >= 32 && static_cast<int64_t>(n_frags) * kc >= 256;
}

hipError_t launch_routed_decode_gate_up(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  const int n_frags = a.N / 32, KT = a.K >> 7;
  const int64_t max_units = static_cast<int64_t>(a.max_tiles) * n_frags;
  int64_t blocks = static_cast<int64_t>(device_cus()) * 4;
  if (blocks > max_units) blocks = max_units;
  if (a.tile_m == 64) return launch_wave<0, 2, 8>(a, n_frags, 1, stream);
  if (KT <= 16) {
    if (use_wave_kernel(a, n_frags, 1))
      return knob(kKnobDecodeVariant) == 1 ? launch_wave<0, 1, 4>(a, n_frags, 1, stream) : launch_wave<0, 1, 8>(a, n_frags, 1, stream);
    routed_stream_kernel<0><<<device_cus() * 2, kDecThreads, 0, stream>>>(a, n_frags, 1);
    return hipGetLastError();
  }
  routed_decode_kernel<0><<<static_cast<unsigned>(blocks), kDecThreads, 0, stream>>>(a, n_frags, 1, (KT + 3) / 4);
  return hipGetLastError();
}

hipError_t launch_routed_decode_down(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  const int n_frags = a.N / 32;
  const int kc = routed_decode_down_planes(a.K);
  if (a.tile_m == 64) return launch_wave<1, 2, 8>(a, n_frags, kc, stream);
  if (use_wave_kernel(a, n_frags, kc))
    return knob(kKnobDecodeVariant) == 1 ? launch_wave<1, 1, 4>(a, n_frags, kc, stream) : launch_wave<1, 1, 8>(a, n_frags, kc, stream);
  routed_stream_kernel<1><<<device_cus() * 3, kDecThreads, 0, stream>>>(a, n_frags, kc);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- shared expert
struct SharedDecodeArgs {
  const uint16_t* act;   // [M, K] bf16
  const uint16_t* w0;    // [N, K] bf16 (gate / down)
  const uint16_t* w1;    // [N, K] bf16 (up)
  int M, N, K;
  uint16_t* h_out;       // gate-up: bf16 [M, N]
  float* y_out;          // down: fp32 partial planes [kc][M, N]
  int64_t plane_stride;
};

// Wave-streaming shared expert for T <= 64: one wavefront = one workgroup owns a 32-channel
// fragment (both matrices in gate-up mode) over its whole K range (a K plane in down mode) and
// streams weight rows AND token rows straight into a private LDS ring of 64-element K steps
// (buffer_load ... lds: a wavefront load covers 8 rows x 128 bytes = whole cache lines, the
// register-operand layout of the MFMA would touch 32 lines per load).  Nothing synchronises:
// the wavefront waits on its own load counter, S-1 steps (48 KiB) stay in flight, which is what
// a few hundred wavefronts need to keep HBM busy.  LDS rows are 128 bytes, chunk XOR-swizzled
// with row bits 1..3 (conflict-free ds_read_b128 of 32 rows).
// wait until at most min(ahead, MAXA) * L of this wavefront's loads are outstanding
template <int L, int MAXA>
__device__ __forceinline__ void wait_steps_ahead(int ahead) {
  if constexpr (MAXA > 0) {
    if (ahead >= MAXA) {
      asm volatile("s_waitcnt vmcnt(%0)" :: "n"(MAXA * L) : "memory");
      return;
    }
    wait_steps_ahead<L, MAXA - 1>(ahead);
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
}

// AL = 1-KiB loads of token rows per K step (8 rows each): 1, 2, 4 or 8 for T <= 8, 16, 32, 64.
// Token rows beyond the batch are never loaded: the MFMA reads whatever the ring holds there
// and the output rows it produces from it are not stored.
template <int MODE, int AL>
struct SharedWaveCfg {
  static constexpr int NMAT = MODE == 0 ? 2 : 1;
  static constexpr int MFR = AL > 4 ? 2 : 1;                // 32-row fragments of tokens
  static constexpr int W_LOADS = NMAT * 4, L = W_LOADS + AL;   // 1-KiB loads per K step
  static constexpr int A_OFF = W_LOADS * 1024;              // token rows follow the weight rows in a slot
  static constexpr int SLOT = L * 1024;                     // only the loaded rows: reads of the other token rows run into the next slot
  static constexpr int TAIL = (MFR * 4 - AL) * 1024;        // ... or, in the last slot, into this much padding
  static constexpr int S_LDS = (65536 - TAIL) / SLOT, S_CNT = 2 + 63 / L;
  static constexpr int S = S_LDS < S_CNT ? S_LDS : S_CNT;   // ring slots: LDS and the 6-bit load counter bound it
  static constexpr int LDS = S * SLOT + TAIL;
};

template <int MODE, int AL>
__global__ __launch_bounds__(64) void shared_wave_kernel(SharedDecodeArgs a, int kc_count, int steps_per_plane) {
  using Cfg = SharedWaveCfg<MODE, AL>;
  constexpr int NMAT = Cfg::NMAT, MFR = Cfg::MFR, L = Cfg::L, SLOT = Cfg::SLOT, S = Cfg::S, A_LOADS = AL;
  constexpr int kBufferFlags = 0x00020000;
  extern __shared__ __attribute__((aligned(16))) unsigned char s_ring[];
  const int M = a.M, N = a.N, K = a.K, KT = K >> 6;
  const int lane = threadIdx.x, r32 = lane & 31, g = lane >> 5;
  // Down projection: workgroup = (32-channel fragment, K plane).  Gate-up (no K planes: the
  // epilogue needs the whole sums): the channels are cut into gridDim.x nearly equal runs of
  // whole quads, at most 32 channels each, so that every CU streams the same number of weight
  // rows (with whole 32-channel fragments 344 workgroups on 256 CUs left a third of the CUs
  // with twice the bytes of the others; a CU serves its requests in order at its share of the
  // HBM bandwidth).  Rows of the fragment past the run are not fetched and not stored.
  const int kc = MODE == 1 ? blockIdx.x % kc_count : 0;
  const int quads = N >> 2;
  const int c0 = MODE == 1 ? (blockIdx.x / kc_count) * 32 : static_cast<int>(static_cast<int64_t>(blockIdx.x) * quads / gridDim.x) * 4;
  const int c1 = MODE == 1 ? c0 + 32 : static_cast<int>(static_cast<int64_t>(blockIdx.x + 1) * quads / gridDim.x) * 4;
  const int step0 = kc * steps_per_plane;
  const int nsteps = min(steps_per_plane, KT - step0);
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)s_ring);
  auto make_rsrc = [&](const void* base, int64_t bytes) {
    const uint64_t p = reinterpret_cast<uint64_t>(base);
    v4i r;
    r.x = static_cast<int>(static_cast<uint32_t>(p));
    r.y = static_cast<int>(static_cast<uint32_t>(p >> 32) & 0xFFFFu);
    r.z = static_cast<int>(bytes);
    r.w = kBufferFlags;
    return r;
  };
  const v4i rsrc_a = make_rsrc(a.act, static_cast<int64_t>(M) * K * 2);
  const v4i rsrc_w0 = make_rsrc(a.w0, static_cast<int64_t>(N) * K * 2);
  const v4i rsrc_w1 = make_rsrc(NMAT == 2 ? a.w1 : a.w0, static_cast<int64_t>(N) * K * 2);
  // load i of a 32-row block covers rows 8i .. 8i+7: lane l lands at row 8i + l/8, physical chunk l%8
  const int ld_row = lane >> 3;
  uint32_t w_voff[4], a_voff[A_LOADS];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int chunk = (lane & 7) ^ ((4 * i + (ld_row >> 1)) & 7);
    const int wrow = c0 + 8 * i + ld_row;
    w_voff[i] = wrow < c1 ? static_cast<uint32_t>(wrow) * static_cast<uint32_t>(K) * 2u + step0 * 128 + chunk * 16
                          : 0x80000000u;   // out of range: nothing is fetched
  }
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int chunk = (lane & 7) ^ ((4 * i + (ld_row >> 1)) & 7);
    a_voff[i] = static_cast<uint32_t>(min(8 * i + ld_row, M - 1)) * static_cast<uint32_t>(K) * 2u + step0 * 128 + chunk * 16;
  }
#define MOTE_DMA(lds_, voff_, rsrc_, soff_)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"           \
               :: "s"(lds_), "v"(voff_), "s"(rsrc_), "s"(soff_) : "memory")
#define MOTE_ISSUE(step_, slot_)                                                                   \
  {                                                                                                \
    const uint32_t base_ = lds0 + (slot_) * SLOT;                                                  \
    const int soff_ = (step_) * 128;                                                               \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) MOTE_DMA(base_ + i * 1024, w_voff[i], rsrc_w0, soff_);            \
    if constexpr (NMAT == 2) {                                                                     \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) MOTE_DMA(base_ + 4096 + i * 1024, w_voff[i], rsrc_w1, soff_);   \
    }                                                                                              \
    _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                            \
      MOTE_DMA(base_ + Cfg::A_OFF + i * 1024, a_voff[i], rsrc_a, soff_);                          \
  }

  v16f acc[NMAT][MFR];
#pragma unroll
  for (int m = 0; m < NMAT; ++m)
#pragma unroll
    for (int f = 0; f < MFR; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[m][f][v] = 0.0f;

  for (int j = 0; j < S - 1 && j < nsteps; ++j) MOTE_ISSUE(j, j);
  const int rd = r32 * 128, sw = (r32 >> 1) & 7;
  int slot = 0, slot_fill = S - 1;
  for (int j = 0; j < nsteps; ++j) {
    // steps j+1 .. min(j+S-2, nsteps-1) may stay in flight
    wait_steps_ahead<L, S - 2>(nsteps - 1 - j);
    const unsigned char* const st = s_ring + slot * SLOT;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const int co = ((2 * s4 + g) ^ sw) << 4;
      bf16x8 af[MFR];
#pragma unroll
      for (int f = 0; f < MFR; ++f) af[f] = *reinterpret_cast<const bf16x8*>(st + Cfg::A_OFF + f * 4096 + rd + co);
#pragma unroll
      for (int m = 0; m < NMAT; ++m) {
        const bf16x8 wf = *reinterpret_cast<const bf16x8*>(st + m * 4096 + rd + co);
#pragma unroll
        for (int f = 0; f < MFR; ++f) acc[m][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, af[f], acc[m][f], 0, 0, 0);
      }
    }
    // refill the slot that was consumed one step ago with step j + S - 1
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (j + S - 1 < nsteps) MOTE_ISSUE(j + S - 1, slot_fill);
    slot_fill = slot;
    slot = slot + 1 == S ? 0 : slot + 1;
  }
#undef MOTE_DMA
#undef MOTE_ISSUE

  // lane l owns token row r32 of every row fragment and channels 8q + 4g .. +3 of the fragment
#pragma unroll
  for (int f = 0; f < MFR; ++f) {
    const int row = f * 32 + r32;
    if (row >= M) continue;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int ch = c0 + 8 * q + 4 * g;
      if (ch >= c1) continue;
      const int64_t o = static_cast<int64_t>(row) * N + ch;
      if constexpr (MODE == 0) {
        uint2 packed;
        packed.x = cvt_pk_bf16(acc[1][f][4 * q] * silu_fast(acc[0][f][4 * q]), acc[1][f][4 * q + 1] * silu_fast(acc[0][f][4 * q + 1]));
        packed.y = cvt_pk_bf16(acc[1][f][4 * q + 2] * silu_fast(acc[0][f][4 * q + 2]), acc[1][f][4 * q + 3] * silu_fast(acc[0][f][4 * q + 3]));
        *reinterpret_cast<uint2*>(a.h_out + o) = packed;
      } else {
        *reinterpret_cast<float4*>(a.y_out + static_cast<int64_t>(kc) * a.plane_stride + o) =
            make_float4(acc[0][f][4 * q], acc[0][f][4 * q + 1], acc[0][f][4 * q + 2], acc[0][f][4 * q + 3]);
      }
    }
  }
}

// ---------------------------------------------------------- quantised shared expert (decode)
// The shared expert with RTN INT8 / INT4 weights (Section 4.3): same wave-streaming scheme as
// shared_wave_kernel, K steps of 64 channels, bf16 token rows, but a weight row of a step is 64
// (INT8) or 32 (INT4) bytes of two's-complement codes in the packed channel order, so a
// 32-row fragment is two / one 1-KiB loads per matrix instead of four.  A lane (row r, K half g)
// reads 16 bytes of its row: INT8 the operands of two MFMAs (K sub-steps 2j, 2j+1), INT4 of all
// four; the codes are sign-extended, converted to fp32 and cut to bf16 (exact: |q| <= 127).  The
// row scales multiply the fp32 sums in the epilogue, so the arithmetic is s_n * sum_c q[n,c] x[c].
struct SharedQDecodeArgs {
  const uint16_t* act;          // [M, K] bf16
  const unsigned char* w0;      // packed codes [N, K*BITS/8] (gate / down)
  const unsigned char* w1;      // (up)
  const float* s0;              // row scales [N]
  const float* s1;
  int M, N, K;
  uint16_t* h_out;
  float* y_out;
  int64_t plane_stride;
};

// NW wavefronts of a workgroup share a channel run and split its K steps (each with a private
// ring), then add their fp32 partial sums through LDS: with one wavefront per workgroup the chain
// of K steps of a wavefront (wait, LDS reads, conversions, MFMAs), not HBM, set the kernel's time.
template <int MODE, int BITS, int AL>
struct SharedQWaveCfg {
  static constexpr int NMAT = MODE == 0 ? 2 : 1;
  static constexpr int MFR = AL > 4 ? 2 : 1;
  static constexpr int NW = AL > 4 ? 2 : 4;                  // wavefronts per workgroup
  static constexpr int WL = BITS == 8 ? 2 : 1;               // 1-KiB loads per matrix and K step
  static constexpr int W_LOADS = NMAT * WL, L = W_LOADS + AL;
  static constexpr int A_OFF = W_LOADS * 1024;
  static constexpr int SLOT = L * 1024;
  static constexpr int TAIL = (MFR * 4 - AL) * 1024;
  static constexpr int S_LDS = ((80 * 1024 - TAIL) / NW) / SLOT, S_CNT = 2 + 63 / L;
  static constexpr int S0 = S_LDS < S_CNT ? S_LDS : S_CNT;
  static constexpr int S = S0 > 8 ? 8 : S0;                  // ring slots per wavefront
  static constexpr int RING = S * SLOT;
  static constexpr int RED = NW * NMAT * MFR * 16 * 64 * 4;  // partial sums of all wavefronts
  static constexpr int LDS = (NW * RING + TAIL) > RED ? (NW * RING + TAIL) : RED;
  static_assert(S >= 2, "at least one K step in flight");
};

// eight consecutive two's-complement codes (bytes of lo/hi, or nibbles of lo) -> bf16x8
template <int BITS>
__device__ __forceinline__ bf16x8 codes_to_bf16(uint32_t lo, uint32_t hi) {
  float f[8];
  if constexpr (BITS == 8) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[i] = static_cast<float>(static_cast<int>(lo << (24 - 8 * i)) >> 24);
      f[4 + i] = static_cast<float>(static_cast<int>(hi << (24 - 8 * i)) >> 24);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = static_cast<float>(static_cast<int>(lo << (28 - 4 * i)) >> 28);
  }
  union { uint32_t u[4]; bf16x8 v; } r;
#pragma unroll
  for (int i = 0; i < 4; ++i)   // small integers: the upper halves of the fp32 patterns are the bf16 values
    r.u[i] = (__float_as_uint(f[2 * i]) >> 16) | (__float_as_uint(f[2 * i + 1]) & 0xFFFF0000u);
  return r.v;
}

template <int MODE, int BITS, int AL>
__global__ __launch_bounds__((64 * SharedQWaveCfg<MODE, BITS, AL>::NW)) void shared_qwave_kernel(SharedQDecodeArgs a, int kc_count,
                                                                                              int steps_per_plane) {
  using Cfg = SharedQWaveCfg<MODE, BITS, AL>;
  constexpr int NMAT = Cfg::NMAT, MFR = Cfg::MFR, L = Cfg::L, SLOT = Cfg::SLOT, S = Cfg::S, A_LOADS = AL, WL = Cfg::WL;
  constexpr int NW = Cfg::NW;
  constexpr int WROW = BITS == 8 ? 64 : 32;        // bytes of a weight row per K step
  constexpr int kBufferFlags = 0x00020000;
  extern __shared__ __attribute__((aligned(16))) unsigned char s_ring[];
  const int M = a.M, N = a.N, K = a.K, KT = K >> 6;
  const int lane = threadIdx.x & 63, r32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kc = MODE == 1 ? blockIdx.x % kc_count : 0;
  const int quads = N >> 2;
  const int c0 = MODE == 1 ? (blockIdx.x / kc_count) * 32 : static_cast<int>(static_cast<int64_t>(blockIdx.x) * quads / gridDim.x) * 4;
  const int c1 = MODE == 1 ? c0 + 32 : static_cast<int>(static_cast<int64_t>(blockIdx.x + 1) * quads / gridDim.x) * 4;
  // K steps of the workgroup, then this wavefront's share of them
  const int wg_step0 = kc * steps_per_plane;
  const int wg_steps = min(steps_per_plane, KT - wg_step0);
  const int per_wave = (wg_steps + NW - 1) / NW;
  const int step0 = wg_step0 + wave * per_wave;
  const int nsteps = max(0, min(per_wave, wg_steps - wave * per_wave));
  unsigned char* const my_ring = s_ring + wave * Cfg::RING;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)my_ring);
  auto make_rsrc = [&](const void* base, int64_t bytes) {
    const uint64_t p = reinterpret_cast<uint64_t>(base);
    v4i r;
    r.x = static_cast<int>(static_cast<uint32_t>(p));
    r.y = static_cast<int>(static_cast<uint32_t>(p >> 32) & 0xFFFFu);
    r.z = static_cast<int>(bytes);
    r.w = kBufferFlags;
    return r;
  };
  const int64_t wrow_bytes = static_cast<int64_t>(K) * BITS / 8;
  const v4i rsrc_a = make_rsrc(a.act, static_cast<int64_t>(M) * K * 2);
  const v4i rsrc_w0 = make_rsrc(a.w0, static_cast<int64_t>(N) * wrow_bytes);
  const v4i rsrc_w1 = make_rsrc(NMAT == 2 ? a.w1 : a.w0, static_cast<int64_t>(N) * wrow_bytes);
  // weight load i of a fragment covers 1024 / WROW rows: lane l lands at LDS byte 16 l of the load,
  // i.e. row l / (WROW/16), chunk l % (WROW/16) -- the fragment sits row-major in LDS
  constexpr int LPR = WROW / 16, RPL = 64 / LPR;   // lanes per row, rows per load
  uint32_t w_voff[WL];
#pragma unroll
  for (int i = 0; i < WL; ++i) {
    const int wrow = c0 + RPL * i + lane / LPR;
    w_voff[i] = wrow < c1 ? static_cast<uint32_t>(wrow) * static_cast<uint32_t>(wrow_bytes) + step0 * WROW + (lane % LPR) * 16
                          : 0x80000000u;   // out of range: nothing is fetched
  }
  const int ld_row = lane >> 3;
  uint32_t a_voff[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int chunk = (lane & 7) ^ ((4 * i + (ld_row >> 1)) & 7);
    a_voff[i] = static_cast<uint32_t>(min(8 * i + ld_row, M - 1)) * static_cast<uint32_t>(K) * 2u + step0 * 128 + chunk * 16;
  }
#define MOTE_DMA(lds_, voff_, rsrc_, soff_)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"           \
               :: "s"(lds_), "v"(voff_), "s"(rsrc_), "s"(soff_) : "memory")
#define MOTE_ISSUE(step_, slot_)                                                                   \
  {                                                                                                \
    const uint32_t base_ = lds0 + (slot_) * SLOT;                                                  \
    _Pragma("unroll") for (int i = 0; i < WL; ++i) MOTE_DMA(base_ + i * 1024, w_voff[i], rsrc_w0, (step_) * WROW);  \
    if constexpr (NMAT == 2) {                                                                     \
      _Pragma("unroll") for (int i = 0; i < WL; ++i) MOTE_DMA(base_ + (WL + i) * 1024, w_voff[i], rsrc_w1, (step_) * WROW);  \
    }                                                                                              \
    _Pragma("unroll") for (int i = 0; i < A_LOADS; ++i)                                            \
      MOTE_DMA(base_ + Cfg::A_OFF + i * 1024, a_voff[i], rsrc_a, (step_) * 128);                  \
  }

  v16f acc[NMAT][MFR];
#pragma unroll
  for (int m = 0; m < NMAT; ++m)
#pragma unroll
    for (int f = 0; f < MFR; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[m][f][v] = 0.0f;

  for (int j = 0; j < S - 1 && j < nsteps; ++j) MOTE_ISSUE(j, j);
  const int rd = r32 * 128, sw = (r32 >> 1) & 7;
  int slot = 0, slot_fill = S - 1;
  for (int j = 0; j < nsteps; ++j) {
    wait_steps_ahead<L, S - 2>(nsteps - 1 - j);
    const unsigned char* const st = my_ring + slot * SLOT;
    // this lane's codes of the step: INT8 two 16-byte reads per matrix (K sub-steps 0,1 and 2,3), INT4 one
    u4 wq[NMAT][WL];
#pragma unroll
    for (int m = 0; m < NMAT; ++m)
#pragma unroll
      for (int i = 0; i < WL; ++i)
        wq[m][i] = *reinterpret_cast<const u4*>(st + m * WL * 1024 + r32 * WROW + (i * 2 + g) * 16);
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const int co = ((2 * s4 + g) ^ sw) << 4;
      bf16x8 af[MFR];
#pragma unroll
      for (int f = 0; f < MFR; ++f) af[f] = *reinterpret_cast<const bf16x8*>(st + Cfg::A_OFF + f * 4096 + rd + co);
#pragma unroll
      for (int m = 0; m < NMAT; ++m) {
        bf16x8 wf;
        if constexpr (BITS == 8) {
          const u4 q = wq[m][s4 >> 1];
          wf = (s4 & 1) ? codes_to_bf16<8>(q.z, q.w) : codes_to_bf16<8>(q.x, q.y);
        } else {
          const u4 q = wq[m][0];
          wf = codes_to_bf16<4>(s4 == 0 ? q.x : s4 == 1 ? q.y : s4 == 2 ? q.z : q.w, 0u);
        }
#pragma unroll
        for (int f = 0; f < MFR; ++f) acc[m][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, af[f], acc[m][f], 0, 0, 0);
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (j + S - 1 < nsteps) MOTE_ISSUE(j + S - 1, slot_fill);
    slot_fill = slot;
    slot = slot + 1 == S ? 0 : slot + 1;
  }
#undef MOTE_DMA
#undef MOTE_ISSUE

  // cross-wavefront reduction: every wavefront parks its partial sums in LDS (the rings are done
  // with), then wavefront w finishes the channel quads q = w, w + NW, ...
  float* const red = reinterpret_cast<float*>(s_ring);
  constexpr int NV = NMAT * MFR * 16;
  __syncthreads();
#pragma unroll
  for (int m = 0; m < NMAT; ++m)
#pragma unroll
    for (int f = 0; f < MFR; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[((wave * NV) + (m * MFR + f) * 16 + v) * 64 + lane] = acc[m][f][v];
  __syncthreads();
#pragma unroll
  for (int f = 0; f < MFR; ++f) {
    const int row = f * 32 + r32;
#pragma unroll
    for (int qq = 0; qq < 4 / NW; ++qq) {
      const int q = wave + qq * NW;
      const int ch = c0 + 8 * q + 4 * g;
      if (row >= M || ch >= c1) continue;
      float sum[NMAT][4];
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float t = 0.0f;
#pragma unroll
          for (int ww = 0; ww < NW; ++ww) t += red[((ww * NV) + (m * MFR + f) * 16 + 4 * q + j) * 64 + lane];   // fixed order
          sum[m][j] = t;
        }
      const int64_t o = static_cast<int64_t>(row) * N + ch;
      const float4 sc0 = *reinterpret_cast<const float4*>(a.s0 + ch);
      if constexpr (MODE == 0) {
        const float4 sc1 = *reinterpret_cast<const float4*>(a.s1 + ch);
        const float gv[4] = {sum[0][0] * sc0.x, sum[0][1] * sc0.y, sum[0][2] * sc0.z, sum[0][3] * sc0.w};
        const float uv[4] = {sum[NMAT - 1][0] * sc1.x, sum[NMAT - 1][1] * sc1.y, sum[NMAT - 1][2] * sc1.z, sum[NMAT - 1][3] * sc1.w};
        uint2 packed;
        packed.x = cvt_pk_bf16(uv[0] * silu_fast(gv[0]), uv[1] * silu_fast(gv[1]));
        packed.y = cvt_pk_bf16(uv[2] * silu_fast(gv[2]), uv[3] * silu_fast(gv[3]));
        *reinterpret_cast<uint2*>(a.h_out + o) = packed;
      } else {
        *reinterpret_cast<float4*>(a.y_out + static_cast<int64_t>(kc) * a.plane_stride + o) =
            make_float4(sum[0][0] * sc0.x, sum[0][1] * sc0.y, sum[0][2] * sc0.z, sum[0][3] * sc0.w);
      }
    }
  }
}

// K planes of the decode down projection: (fragments x planes) workgroups should fill two
// slots per CU evenly, with planes of at least 8 K steps of 64.  The second value is the plane length.
static void shared_decode_down_split(int d, int K, int* kc_out, int* steps_out) {
  const int KT = K >> 6, n_frags = d / 32;
  int kc = (device_cus() * 2 + n_frags / 2) / (n_frags > 0 ? n_frags : 1);
  if (kc > KT / 8) kc = KT / 8;
  if (kc < 1) kc = 1;
  const int steps = (KT + kc - 1) / kc;
  *kc_out = (KT + steps - 1) / steps;
  *steps_out = steps;
}

int shared_decode_down_planes(int d, int K) {
  int kc, steps;
  shared_decode_down_split(d, K, &kc, &steps);
  return kc;
}


template <int MODE, int AL>
static hipError_t launch_shared_wave_al(const SharedDecodeArgs& a, int n_frags, int kc, int steps_per_plane, hipStream_t stream) {
  constexpr int lds = SharedWaveCfg<MODE, AL>::LDS;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(shared_wave_kernel<MODE, AL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  shared_wave_kernel<MODE, AL><<<n_frags * kc, 64, lds, stream>>>(a, kc, steps_per_plane);
  return hipGetLastError();
}

template <int MODE>
static hipError_t launch_shared_wave(const SharedDecodeArgs& a, int n_frags, int kc, int steps_per_plane, hipStream_t stream) {
  if (a.M <= 8) return launch_shared_wave_al<MODE, 1>(a, n_frags, kc, steps_per_plane, stream);
  if (a.M <= 16) return launch_shared_wave_al<MODE, 2>(a, n_frags, kc, steps_per_plane, stream);
  if (a.M <= 32) return launch_shared_wave_al<MODE, 4>(a, n_frags, kc, steps_per_plane, stream);
  return launch_shared_wave_al<MODE, 8>(a, n_frags, kc, steps_per_plane, stream);
}

hipError_t launch_shared_decode_gate_up(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up, int T, int d,
                                        int F, uint16_t* h_s, hipStream_t stream) {
  SharedDecodeArgs a{x, w_gate, w_up, T, F, d, h_s, nullptr, 0};
  const int n_frags = F / 32, KT = d >> 6;
  // channel runs instead of fragments: see the kernel
  const int runs = std::max(device_cus() * 2, n_frags);
  return launch_shared_wave<0>(a, std::min(runs, F / 4), 1, KT, stream);
}

template <int MODE, int BITS, int AL>
static hipError_t launch_shared_qwave_al(const SharedQDecodeArgs& a, int n_blocks, int kc, int steps_per_plane, hipStream_t stream) {
  constexpr int lds = SharedQWaveCfg<MODE, BITS, AL>::LDS;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(shared_qwave_kernel<MODE, BITS, AL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  shared_qwave_kernel<MODE, BITS, AL><<<n_blocks, 64 * SharedQWaveCfg<MODE, BITS, AL>::NW, lds, stream>>>(a, kc, steps_per_plane);
  return hipGetLastError();
}

template <int MODE, int BITS>
static hipError_t launch_shared_qwave(const SharedQDecodeArgs& a, int n_blocks, int kc, int steps_per_plane, hipStream_t stream) {
  if (a.M <= 8) return launch_shared_qwave_al<MODE, BITS, 1>(a, n_blocks, kc, steps_per_plane, stream);
  if (a.M <= 16) return launch_shared_qwave_al<MODE, BITS, 2>(a, n_blocks, kc, steps_per_plane, stream);
  if (a.M <= 32) return launch_shared_qwave_al<MODE, BITS, 4>(a, n_blocks, kc, steps_per_plane, stream);
  return launch_shared_qwave_al<MODE, BITS, 8>(a, n_blocks, kc, steps_per_plane, stream);
}

hipError_t launch_shared_q_decode_gate_up(const uint16_t* x, const void* w_gate, const void* w_up, const float* s_gate,
                                          const float* s_up, int bits, int T, int d, int F, uint16_t* h_s,
                                          hipStream_t stream) {
  SharedQDecodeArgs a{x, static_cast<const unsigned char*>(w_gate), static_cast<const unsigned char*>(w_up), s_gate, s_up,
                      T, F, d, h_s, nullptr, 0};
  const int n_frags = F / 32, KT = d >> 6;
  const int runs = std::min(std::max(device_cus() * 2, n_frags), F / 4);
  return bits == 8 ? launch_shared_qwave<0, 8>(a, runs, 1, KT, stream) : launch_shared_qwave<0, 4>(a, runs, 1, KT, stream);
}

hipError_t launch_shared_q_decode_down(const uint16_t* h_s, const void* w_down, const float* s_down, int bits, int T,
                                       int d, int F, float* y_s, hipStream_t stream) {
  SharedQDecodeArgs a{h_s, static_cast<const unsigned char*>(w_down), nullptr, s_down, nullptr, T, d, F, nullptr, y_s,
                      static_cast<int64_t>(T) * d};
  const int n_frags = d / 32;
  int kc, steps;
  shared_decode_down_split(d, F, &kc, &steps);
  return bits == 8 ? launch_shared_qwave<1, 8>(a, n_frags * kc, kc, steps, stream)
                   : launch_shared_qwave<1, 4>(a, n_frags * kc, kc, steps, stream);
}

hipError_t launch_shared_decode_down(const uint16_t* h_s, const uint16_t* w_down, int T, int d, int F, float* y_s,
                                     hipStream_t stream) {
  SharedDecodeArgs a{h_s, w_down, nullptr, T, d, F, nullptr, y_s, static_cast<int64_t>(T) * d};
  const int n_frags = d / 32;
  int kc, steps;
  shared_decode_down_split(d, F, &kc, &steps);
  return launch_shared_wave<1>(a, n_frags, kc, steps, stream);
}

}  // namespace mote
