// Grouped ternary GEMMs of the routed experts (Eq.5-6, and the ternary linear layer
// Y = Q_w(W) Q_a(x) at the end of Section 3.1) on int8 MFMA with int32 accumulation.
//
//   gate-up mode : G = t_gate . q_x, U = t_up . q_x for the rows of one expert, then the
//                  fused epilogue  h = bf16( (U*s_u) * SiLU(G*s_g) ),  s = beta_x/127 * alpha
//   down mode    : D = t_down . q_h, stored as int32 (the combine kernel applies the scales)
//
// Work decomposition: the dispatch plan lists row tiles (one expert each, BM rows); a
// workgroup owns one row tile x one block of BN output channels and walks K in steps of
// 128.  Activations (int8, gathered through tok_of in gate-up mode) are loaded straight
// into LDS (global_load_lds), 16-byte chunks XOR-swizzled by row so that ds_read_b128 of
// 32 consecutive rows is conflict free; three stages, requested two K steps ahead.
// Packed weights take the same road (global -> LDS directly, ring of three stages) and stay
// packed in LDS: a tile of 32 rows x 128 channels is 1 KiB = one 16-byte LDS read per lane,
// each 32-bit word expands in registers with (w >> 2j) & 0x03030303 into the four operand
// registers of one v_mfma_i32_32x32x32_i8.  The codes are t+1, so the accumulator holds
// sum (t+1) q; it starts at minus the row sum of q.
//
// MFMA operand mapping (32x32x32 i8): first operand = weights, lane l supplies output
// channel l%32 and 16 consecutive input channels of half l/32; second operand =
// activations, lane l supplies dispatch row l%32 and the same 16 channels.  Result register
// v of lane l is output channel 8*(v/4) + 4*(l/32) + v%4 of dispatch row l%32.
//
// Epilogue: every wavefront transposes its result fragments through a private LDS patch so
// that a global store instruction covers whole rows of a 32-row block.
#include <stdlib.h>

#include <algorithm>
#include <type_traits>
#include "common.h"
#include "launch.h"

namespace mote {

template <int MODE_, int BM_W_, int BN_W_, int WAVES_M_, int WAVES_N_, int MIN_BLOCKS_ = 1>
struct RoutedCfg {
  static constexpr int MODE = MODE_;  // 0 gate-up (two matrices, SwiGLU epilogue), 1 down
  static constexpr int NMAT = MODE_ == 0 ? 2 : 1;
  static constexpr int BM_W = BM_W_, BN_W = BN_W_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int MIN_BLOCKS = MIN_BLOCKS_;  // wavefronts per SIMD the register budget must allow (2 workgroups per CU)
  static constexpr int BM = 32 * BM_W_ * WAVES_M_;
  static constexpr int BN = 32 * BN_W_ * WAVES_N_;
  static constexpr int WAVES = WAVES_M_ * WAVES_N_;
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int ROWS_PER_PASS = THREADS / 8;
  static constexpr int A_PASSES = BM / ROWS_PER_PASS;
  static constexpr int A_BYTES = BM * 128;                       // int8 activation tile of one K step
  static constexpr int W_FRAGS = NMAT * BN / 32;                 // packed 1-KiB weight fragments of one K step
  static constexpr int W_PER_WAVE = W_FRAGS / WAVES;
  static constexpr int STAGE_BYTES = A_BYTES + W_FRAGS * 1024;
  // epilogue patch of one wavefront: 32 rows x PATCH_F fragments of 32 outputs + 16 bytes of row padding
  static constexpr int OUT_BYTES = MODE_ == 0 ? 2 : 4;
  static constexpr int PATCH_F = MODE_ == 0 ? BN_W_ : 1;
  static constexpr int PATCH_ROW = PATCH_F * 32 * OUT_BYTES + 16;
  static constexpr int PATCH_BYTES = 32 * PATCH_ROW;
  static_assert(BM % ROWS_PER_PASS == 0, "activation loader covers the tile in whole passes");
  static_assert(W_FRAGS % WAVES == 0, "every wavefront requests the same number of weight fragments");
  static_assert(64 % (PATCH_F * 32 * OUT_BYTES / 16) == 0, "an epilogue read covers whole rows");
};

#ifdef MOTE_TRACE
__device__ unsigned long long g_trace[1024 * 32 * 8];
#define MOTE_TP(k_) if (Cfg::MODE == MOTE_TRACE && tid == 0 && tile_it < 32) g_trace[(blockIdx.x * 32 + tile_it) * 8 + (k_)] = __builtin_readcyclecounter();
#else
#define MOTE_TP(k_)
#endif

// LDS tile geometry: 128-byte rows of eight 16-byte chunks, chunk index XOR-swizzled with
// bits 1..3 of the row.  Two consecutive rows span the 64 banks once, so 16 lanes that read
// the same chunk of 16 consecutive rows (one quarter of a ds_read_b128) hit 16 distinct
// 4-bank groups: conflict free (measured 2x faster than swizzling with row bits 0..2).
__device__ __forceinline__ int lds_a_offset(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

// One 128-channel K step of a wavefront is four 32-channel sub-steps; each reads BM_W
// activation fragments from LDS and, per weight fragment, unpacks 16 codes per lane and feeds
// BM_W MFMAs (MOTE_KSTEP in the kernel).  The global loads of a later K step are spread over
// the four sub-steps: issued in one burst right after the barrier, eight wavefronts x eight
// 1-KiB loads fill the CU's vector-memory queue and every wavefront stalls in issue (measured:
// about 800 cycles per K step) before it reaches its first MFMA.
constexpr int kFixedShares = 1 << 20;   // n_static from which every tile of a workgroup is fixed

// SKIP_: what a partly filled row tile (the last one of an expert, half empty on average) saves.
//   2: every 32-row fragment that holds no rows is neither read nor contracted.  The conditions
//      cost full tiles about 8 % (scalar branches between the MFMAs), so this variant is launched
//      only when most row tiles are partly filled (few rows per expert).
//   1: only a wavefront whose whole block of rows is empty idles through the K steps (it still
//      issues its share of the loads and meets the barriers): one scalar branch per K step.
template <typename Cfg, int SKIP_>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_BLOCKS) void routed_gemm_kernel(RoutedGemmArgs a, int n_ntiles, int kplanes, int ktp, int group_m, int n_static) {
  constexpr int NMAT = Cfg::NMAT, BM_W = Cfg::BM_W, BN_W = Cfg::BN_W;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, THREADS = Cfg::THREADS;
  constexpr int A_BYTES = Cfg::A_BYTES, STAGE_BYTES = Cfg::STAGE_BYTES;
  constexpr bool SKIP = SKIP_ == 2;                 // fragment-level tests inside the K loop
  constexpr int NB = BN / 32;                       // 32-channel blocks of the tile
  constexpr int W_PER_WAVE = Cfg::W_PER_WAVE;       // weight fragments a wavefront requests per K step
  constexpr int NLOAD = Cfg::A_PASSES + W_PER_WAVE; // vector-memory operations a wavefront issues per K step
  static_assert(BM <= THREADS, "one thread per tile row publishes the row metadata");
  static_assert((Cfg::WAVES == 4 || Cfg::WAVES == 8) && Cfg::ROWS_PER_PASS == 8 * Cfg::WAVES, "a loader pass is 8 rows per wavefront");
  static_assert(NLOAD < 16, "fits the low vmcnt field");
  __shared__ __attribute__((aligned(16))) unsigned char s_lds[3 * STAGE_BYTES];
  __shared__ float s_beta[2][BM];   // row metadata (absmax, integer row sum), double buffered by tile parity
  __shared__ int s_rs[2][BM];

  const int K = a.K, N = a.N;
  const int KT = K >> 7;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int r32 = lane & 31, g = lane >> 5;
  const int a_row_base = wm * BM_W * 32 + r32;
  const int64_t expert_words = static_cast<int64_t>(N) * K / 16;
  // LDS byte address of the stage area (what M0 takes for a direct-to-LDS load)
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)s_lds);

  // Persistent workgroups: the grid is one wave of resident workgroups that take (row tile,
  // channel tile) pairs until none is left.  Workgroups are dealt to the 8 XCDs round-robin by
  // linear id; XCD x owns the list of the channel tiles x, x+8, ... (or, when there are fewer
  // than 16 channel tiles, of the row tiles x, x+8, ...).  Inside a list the pairs are ordered in
  // bands of group_m row tiles, row tile fastest: the workgroups resident at one time then
  // cover about group_m row tiles x (resident / group_m) channel tiles, so every activation
  // tile and every weight slice fetched into that XCD's L2 is used by several of them.
  // With kplanes > 1 (down projection of small problems) the contraction is cut into planes
  // of ktp K steps; a (channel tile, plane) pair then plays the role of a channel tile and each
  // plane writes its own partial output that the combine kernel adds.
  //
  // The first n_static pairs of a workgroup are fixed (list positions b, b + stride, ... of its
  // own XCD); every later one is drawn from a counter per list (plan.sched, one cache line each,
  // zeroed by the dispatch plan kernel), first from the own XCD's list and, once that is empty,
  // from the others'.  Two workgroups share a CU and the hardware favours the older one: with
  // fixed shares only, the favoured half of the grid finished its tiles at 60 % of the kernel's
  // time (measured, 23 tiles per workgroup) and the other half ran the rest alone, one
  // workgroup per CU.  A draw is a device-wide atomic that costs microseconds when the whole
  // grid draws at once, so problems of a few tiles per workgroup keep fixed shares
  // (n_static = kAllStatic).
  //
  // With fixed shares the last round of a list is often nearly empty (C3 down projection: 136
  // pairs on 64 workgroups, so 8 workgroups ran a third tile while 56 idled: 40 % of the
  // kernel's time).  If at most half of the workgroups would have a pair in that round, each
  // pair of the round is cut into up to a.split_max K planes that go to different workgroups
  // (measured 316 -> 299 us; the favoured workgroups of the first rounds still finish early.
  // Cutting the last pairs of drawn lists the same way was slower: the combine kernel then adds
  // four planes for a quarter of the rows);
  // plane kc writes partial plane kc of the output, and the pair's plane count goes into the
  // rows' words of plan.row_planes (2 bits per channel tile, hence at most 16 channel tiles)
  // for the combine kernel (down projection with a single uniform plane only).
  // A ticket packs list (3 bits), planes of the pair (3), plane (2) and the slot in the list.
  n_ntiles *= kplanes;
  const int own = blockIdx.x & 7;
  const int n_mtiles = load_uniform(a.plan.n_tiles);
  const bool split_n = n_ntiles >= 16;
  const int stride = gridDim.x >> 3;
  auto list_ntiles = [&](int x) { return split_n ? (n_ntiles - x + 7) >> 3 : n_ntiles; };
  auto list_mtiles = [&](int x) { return split_n ? n_mtiles : (n_mtiles - x + 7) >> 3; };
  // When the lists are short, their uneven lengths (whole row or channel tiles per XCD) can cost
  // a whole extra round of tiles; the pairs are then dealt to the XCDs one by one instead
  // (pair p = row tile * n_ntiles + channel tile goes to list p % 8).
  const int n_pairs = n_mtiles * n_ntiles;
  const int band_longest = (split_n ? ((n_ntiles + 7) >> 3) * n_mtiles : ((n_mtiles + 7) >> 3) * n_ntiles);
  const bool flat = (((n_pairs + 7) >> 3) + stride - 1) / stride < (band_longest + stride - 1) / stride;
  auto list_work = [&](int x) { return flat ? (n_pairs - x + 7) >> 3 : list_ntiles(x) * list_mtiles(x); };
  int32_t* const sched = a.plan.sched + (Cfg::MODE == 0 ? 0 : 8 * kSchedStride);
  // thread 0's scheduler state: 0 = the own list may still have pairs, 1 = take from the other lists, 8 = all empty
  __shared__ int s_sched[1];
  auto make_ticket = [](int slot, int x, int kc, int planes) { return (slot << 8) | (kc << 6) | (planes << 3) | x; };
  const bool may_split = Cfg::MODE == 1 && kplanes == 1 && n_ntiles <= 16;
  // Thread 0 only.  One draw from the own list while it lasts; afterwards a look at all eight
  // counters picks a list that still has pairs (one round trip even when every list is empty).
  auto fetch_ticket = [&](int& cur) -> int {
    if (cur == 0) {
      const int sl = n_static * stride + __hip_atomic_fetch_add(sched + own * kSchedStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (sl < list_work(own)) return make_ticket(sl, own, 0, 1);
      cur = 1;
    }
    while (cur < 8) {
      int seen[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) seen[i] = __hip_atomic_load(sched + i * kSchedStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      int pick = -1;
#pragma unroll
      for (int i = 7; i >= 1; --i) {
        const int x = (own + i) & 7;
        int c = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) c = j == x ? seen[j] : c;
        if (n_static * stride + c < list_work(x)) pick = x;
      }
      if (pick < 0) { cur = 8; break; }
      const int sl = n_static * stride + __hip_atomic_fetch_add(sched + pick * kSchedStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (sl < list_work(pick)) return make_ticket(sl, pick, 0, 1);
    }
    return -1;
  };
  // ticket of this workgroup's j-th tile (thread 0 only)
  auto next_ticket = [&](int& cur, int j) -> int {
    if (j < n_static) {
      const int b = blockIdx.x >> 3;
      const int w = list_work(own);
      const int full = w / stride, last = w - full * stride;   // whole rounds, pairs of the last partial round
      if (j < full) return make_ticket(b + j * stride, own, 0, 1);
      if (j == full && last > 0) {
        int planes = 1;
        if (may_split && n_static >= kFixedShares && 2 * last <= stride)
          planes = max(1, min(min(a.split_max, stride / last), KT >> 3));
        if (b < last * planes) return make_ticket(full * stride + b / planes, own, b % planes, planes);
      }
      if (cur == 0) cur = 1;   // the own list ends within its fixed part
    }
    return fetch_ticket(cur);
  };
  __shared__ int s_ticket[2];   // ticket of tile i lives in s_ticket[i & 1]
  if (tid == 0) {
    // list 0 is the longest: if it ends within the fixed pairs there is nothing to draw anywhere
    int cur = list_work(0) <= n_static * stride ? 8 : 0;
    s_ticket[0] = next_ticket(cur, 0);
    s_sched[0] = cur;
  }
  __syncthreads();
  int ticket = __builtin_amdgcn_readfirstlane(s_ticket[0]);
  if (ticket < 0) return;
  int tile_i = 0;

  // Loader.  Both operands travel global -> LDS directly (buffer_load ... lds, 16 bytes per
  // lane, no register holds bytes in flight) into one of three stages, two K steps ahead of
  // the MFMAs that consume them.
  //   activations: a wavefront load fills 8 consecutive 128-byte tile rows; lane l lands at
  //     byte 16*l of that 1-KiB block, so the XOR swizzle is applied on the global side (lane l
  //     fetches chunk (l&7) ^ swizzle(row));
  //   weights: a packed 32-channel x 128 fragment is 1 KiB = one wavefront load, stored as is.
  // The loads are written in assembly: the compiler has no exact model of outstanding
  // direct-to-LDS loads across this loop's control flow and would drain the queue before the
  // LDS reads of every K step.  Vector-memory operations complete in issue order, so waiting
  // for "all but the NLOAD youngest" retires the K step that is about to be contracted while
  // the following one stays in flight; anything else the wavefront has issued since (stores of
  // the previous epilogue, gather loads) only makes that wait stricter.
  constexpr int kBufferFlags = 0x00020000;   // raw buffer, 32-bit data format
  v4i rsrc_q;
  {
    const uint64_t p = reinterpret_cast<uint64_t>(a.q);
    rsrc_q.x = static_cast<int>(static_cast<uint32_t>(p));
    rsrc_q.y = static_cast<int>(static_cast<uint32_t>(p >> 32) & 0xFFFFu);
    rsrc_q.z = static_cast<int>(a.q_rows * K);
    rsrc_q.w = kBufferFlags;
  }
  v4i rsrc_meta;                           // beta (wavefronts 0 and 1) or rowsum (2 and 3): one 4-byte value per row of q
  {
    const uint64_t p = wave_u < 2 ? reinterpret_cast<uint64_t>(a.beta) : reinterpret_cast<uint64_t>(a.rowsum);
    rsrc_meta.x = static_cast<int>(static_cast<uint32_t>(p));
    rsrc_meta.y = static_cast<int>(static_cast<uint32_t>(p >> 32) & 0xFFFFu);
    rsrc_meta.z = static_cast<int>(a.q_rows * 4);
    rsrc_meta.w = kBufferFlags;
  }
  v4i rsrc_w[W_PER_WAVE];                  // the expert's packed matrix each of this wavefront's fragments lives in
  uint32_t w_soff[W_PER_WAVE];             // uniform: byte offset of that fragment's first tile in the plane
  uint32_t a_off[Cfg::A_PASSES];           // byte offset of this lane's 16 bytes inside q, K step 0 of the plane
  const uint32_t w_lane = lane * 16;
  const uint32_t a_chunk = static_cast<uint32_t>(((tid & 7) ^ ((tid >> 4) & 7)) << 4);
  int src_row[Cfg::A_PASSES];   // row of q (gathered) per loader pass, next tile
  int meta_row = 0;             // row of q whose beta (wavefronts 0-1) or row sum (2-3) this lane requests
  int mt, nt, kc, expert, row0, rows, ktl, ktp_t, planes_t;   // ktp_t: K steps per plane of this tile, planes_t: its planes
  int par = 0;
  int st_cur = 0, st_nxt = STAGE_BYTES, st_nx2 = 2 * STAGE_BYTES;   // stage of K step kt, kt+1, kt+2 (byte offsets)

#define MOTE_DECODE(ticket_, mt_, nt_, kc_, ktp_, planes_)                      \
  {                                                                             \
    const int x_ = (ticket_) & 7, slot_ = (ticket_) >> 8;                       \
    planes_ = ((ticket_) >> 3) & 7;                                             \
    int ntk_;                                                                   \
    if (flat) {                                                                 \
      const int p_ = slot_ * 8 + x_;                                            \
      mt_ = p_ / n_ntiles;                                                      \
      ntk_ = p_ - mt_ * n_ntiles;                                               \
    } else {                                                                    \
      const int xm_ = list_mtiles(x_);                                          \
      const int per_group_ = group_m * list_ntiles(x_);                         \
      const int grp_ = slot_ / per_group_;                                      \
      const int in_ = slot_ - grp_ * per_group_;                                \
      const int gsz_ = min(xm_ - grp_ * group_m, group_m);                      \
      const int ni_ = in_ / gsz_, mi_ = grp_ * group_m + (in_ - ni_ * gsz_);    \
      mt_ = split_n ? mi_ : x_ + 8 * mi_;                                       \
      ntk_ = split_n ? x_ + 8 * ni_ : ni_;                                      \
    }                                                                           \
    if (kplanes > 1) {                                                          \
      nt_ = ntk_ / kplanes;                                                     \
      kc_ = ntk_ - nt_ * kplanes;                                               \
      ktp_ = ktp;                                                               \
    } else {                                                                    \
      nt_ = ntk_;                                                               \
      kc_ = ((ticket_) >> 6) & 3;                                               \
      ktp_ = (KT + planes_ - 1) / planes_;                                      \
    }                                                                           \
  }
  // gate-up rows are gathered through tok_of (a.gather), down rows are the dispatch rows themselves
#define MOTE_GATHER(row0_, rows_)                                                                  \
  {                                                                                                \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p) {                                    \
      const int rslot_ = (row0_) + min(p * Cfg::ROWS_PER_PASS + (tid >> 3), (rows_)-1);            \
      if constexpr (Cfg::MODE == 0) src_row[p] = a.gather[rslot_];                                 \
      else src_row[p] = rslot_;                                                                    \
    }                                                                                              \
    const int mslot_ = (row0_) + min(tid & (BM - 1), (rows_)-1);                                   \
    if constexpr (Cfg::MODE == 0) meta_row = a.gather[mslot_];                                     \
    else meta_row = mslot_;                                                                        \
  }
  // Fragment ids of a stage: matrix m, channel block cb -> m*NB + cb.  Wavefront w requests the
  // ids w*W_PER_WAVE ... ; every wavefront later reads the ids of its own channel blocks.
#define MOTE_POINTERS(expert_, nt_, kc_, ktp_)                                                           \
  {                                                                                                \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                                      \
      a_off[p] = static_cast<uint32_t>(src_row[p]) * static_cast<uint32_t>(K) + a_chunk +          \
                 static_cast<uint32_t>((kc_) * (ktp_)) * 128u;                                        \
    _Pragma("unroll") for (int i = 0; i < W_PER_WAVE; ++i) {                                       \
      const int fid_ = wave_u * W_PER_WAVE + i;                                                    \
      const int m_ = fid_ / NB, cb_ = fid_ - m_ * NB;                                              \
      const int n_frag_ = (nt_) * BN + cb_ * 32;                                                   \
      const int nt32_ = (n_frag_ < N ? n_frag_ : 0) >> 5; /* fragments past N read tile 0 */       \
      w_soff[i] = static_cast<uint32_t>(nt32_ * KT + (kc_) * (ktp_)) * 1024u;                         \
      const uint32_t* mat_ = (NMAT == 2 && m_ == 1) ? a.w_up : a.w_gate;                           \
      const uint64_t p_ = reinterpret_cast<uint64_t>(mat_ + static_cast<int64_t>(expert_) * expert_words); \
      rsrc_w[i].x = static_cast<int>(static_cast<uint32_t>(p_));                                   \
      rsrc_w[i].y = static_cast<int>(static_cast<uint32_t>(p_ >> 32) & 0xFFFFu);                   \
      rsrc_w[i].z = static_cast<int>(expert_words * 4);                                            \
      rsrc_w[i].w = kBufferFlags;                                                                  \
    }                                                                                              \
  }
  // one 16-byte-per-lane direct load: LDS byte address (uniform), lane offset, buffer, scalar offset.
  // M0 is written inside the statement and not listed as a clobber: the AMDGPU backend reserves M0
  // (it never keeps a value of its own there across instructions; it writes M0 itself directly
  // before each instruction of its own that reads it), and it rejects reserved registers in clobber
  // lists with a warning.  The same holds for the other direct-load statements of this library.
#define MOTE_DMA(lds_, voff_, rsrc_, soff_)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"           \
               :: "s"(lds_), "v"(voff_), "s"(rsrc_), "s"(soff_) : "memory")
#define MOTE_DMA_A(stage_, ks_, p_)                                                                \
  MOTE_DMA(lds0 + (stage_) + ((p_) * Cfg::ROWS_PER_PASS + wave_u * 8) * 128, a_off[p_], rsrc_q, (ks_) * 128)
#define MOTE_DMA_W(stage_, ks_, i_)                                                                \
  MOTE_DMA(lds0 + (stage_) + A_BYTES + (wave_u * W_PER_WAVE + (i_)) * 1024, w_lane, rsrc_w[i_],    \
           w_soff[i_] + (ks_) * 1024)
  // Row metadata of a tile into the parity buffer par_: lane l of wavefront 0/1 brings beta of
  // tile row 64*w + l, of wavefront 2/3 the row sum of tile row 64*(w-2) + l (4 bytes per lane).
  // Issued before the tile's first K step, so the wait for that step covers it.
#define MOTE_DMA_META(par_)                                                                        \
  if (wave_u < 4) {                                                                                \
    const uint32_t dst_ = wave_u < 2                                                               \
        ? (uint32_t)(uintptr_t)((__attribute__((address_space(3))) float*)&s_beta[par_][wave_u * 64]) \
        : (uint32_t)(uintptr_t)((__attribute__((address_space(3))) int*)&s_rs[par_][(wave_u - 2) * 64]); \
    const uint32_t voff_ = static_cast<uint32_t>(meta_row) * 4u;                                   \
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"           \
                 :: "s"(dst_), "v"(voff_), "s"(rsrc_meta) : "memory");                             \
  }
  // all loads of one K step at once (tile start)
#define MOTE_ISSUE_STEP(stage_, ks_)                                                               \
  {                                                                                                \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p) MOTE_DMA_A(stage_, ks_, p);          \
    _Pragma("unroll") for (int i = 0; i < W_PER_WAVE; ++i) MOTE_DMA_W(stage_, ks_, i);             \
  }
  // in_flight_: whether the loads of one more K step were issued after the ones needed now
#define MOTE_WAIT_BARRIER(in_flight_)                                                              \
  {                                                                                                \
    if (in_flight_) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NLOAD) : "memory");                  \
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                          \
    asm volatile("s_barrier" ::: "memory");                                                        \
  }

  // ---- first tile: the whole dependent chain (plan -> gather -> rows) is paid once ----
  MOTE_DECODE(ticket, mt, nt, kc, ktp_t, planes_t);
  expert = load_uniform(a.plan.tile_expert + mt);
  row0 = load_uniform(a.plan.tile_row0 + mt);
  rows = load_uniform(a.plan.tile_rows + mt);
  ktl = min(ktp_t, KT - kc * ktp_t);
  MOTE_GATHER(row0, rows);
  MOTE_POINTERS(expert, nt, kc, ktp_t);
  MOTE_DMA_META(0);
  MOTE_ISSUE_STEP(st_cur, 0);
  if (ktl > 1) MOTE_ISSUE_STEP(st_nxt, 1);
  if (tid == 0) {   // second ticket, drawn while the first loads travel
    int cur = s_sched[0];
    const int t = next_ticket(cur, 1);
    s_sched[0] = cur;
    s_ticket[1] = t;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }

#ifdef MOTE_TRACE
  int tile_it = 0;
#endif
  for (;;) {
    MOTE_TP(0)
#ifdef MOTE_TRACE
    if (Cfg::MODE == MOTE_TRACE && tid == 0 && tile_it < 32) g_trace[(blockIdx.x * 32 + tile_it) * 8 + 6] = wall_clock64();
#endif
    MOTE_WAIT_BARRIER(ktl > 1);   // K step 0 (and the metadata) visible to every wavefront; so is the next ticket
    // (1) coordinates of the next tile of this workgroup (uniform scalar loads)
    const int nticket = __builtin_amdgcn_readfirstlane(s_ticket[(tile_i + 1) & 1]);
    const bool has_next = nticket >= 0;
    int mt2 = mt, nt2 = nt, kc2 = kc, expert2 = expert, row02 = row0, rows2 = rows, ktp2 = ktp_t, planes2 = planes_t;
    if (has_next) {
      MOTE_DECODE(nticket, mt2, nt2, kc2, ktp2, planes2);
      expert2 = load_uniform(a.plan.tile_expert + mt2);
      row02 = load_uniform(a.plan.tile_row0 + mt2);
      rows2 = load_uniform(a.plan.tile_rows + mt2);
    }
    MOTE_TP(1)
    const int n_wave0 = nt * BN + wn * BN_W * 32;  // first output channel of this wavefront
    const float al0 = load_uniform(a.alpha + expert * 3 + (Cfg::MODE == 0 ? 0 : 2));
    const float al1 = Cfg::MODE == 0 ? load_uniform(a.alpha + expert * 3 + 1) : 0.0f;

    // Accumulators start at -rowsum(q): the stored codes are t+1, so sum (t+1) q - sum q = sum t q.
    v16i acc[NMAT][BM_W][BN_W];
#pragma unroll
    for (int i = 0; i < BM_W; ++i) {
      const int nrs = kc == 0 ? -s_rs[par][wm * BM_W * 32 + i * 32 + r32] : 0;   // the correction enters plane 0 only
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < BN_W; ++f)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[m][i][f][v] = nrs;
    }
    // row gather of the next tile: the indices are in registers when the K loop ends
    if (has_next) MOTE_GATHER(row02, rows2);
    // Rows of this wavefront's block that exist: the last row tile of an expert is half empty on
    // average, and a 32-row fragment without rows is neither read nor contracted (its MFMA slots go
    // to the other wavefronts of the SIMD).  Wavefront-uniform, so these are scalar branches.
    const int rows_w = SKIP_ != 0 ? __builtin_amdgcn_readfirstlane(rows - (wave_u % Cfg::WAVES_M) * BM_W * 32) : BM_W * 32;

    // (2) K loop.  K step kt contracts stage st_cur while the loads of kt+2 are issued, one
    // quarter of them per 32-channel sub-step (a burst of loads right after the barrier fills
    // the CU's vector-memory queue and stalls every wavefront in issue), into the stage that the
    // barrier at the end of step kt-1 released.
    const int ktl_mm = (SKIP_ == 1 && rows_w <= 0) ? 0 : ktl;   // a wavefront without rows contracts nothing ...
    for (int kt = 0; kt < ktl - ktl_mm; ++kt) {                  // ... it only issues its share of the loads and meets the barriers
      const bool pf = kt + 2 < ktl;
      if (pf) {
#pragma unroll
        for (int p = 0; p < Cfg::A_PASSES; ++p) MOTE_DMA_A(st_nx2, kt + 2, p);
#pragma unroll
        for (int i = 0; i < W_PER_WAVE; ++i) MOTE_DMA_W(st_nx2, kt + 2, i);
      }
      MOTE_WAIT_BARRIER(pf);
      const int t = st_cur; st_cur = st_nxt; st_nxt = st_nx2; st_nx2 = t;
    }
    for (int kt = 0; kt < ktl_mm; ++kt) {
      const bool pf = kt + 2 < ktl;
      const unsigned char* const st = s_lds + st_cur;
      u4 wf[NMAT][BN_W];
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < BN_W; ++f)
          wf[m][f] = *reinterpret_cast<const u4*>(st + A_BYTES + (m * NB + wn * BN_W + f) * 1024 + w_lane);
      v4i af[2][BM_W];
#pragma unroll
      for (int i = 0; i < BM_W; ++i)
        if (!SKIP || i * 32 < rows_w) af[0][i] = *reinterpret_cast<const v4i*>(st + lds_a_offset(a_row_base + i * 32, g));
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (pf) {   // quarter s of the loads of K step kt+2
#pragma unroll
          for (int p = 0; p < Cfg::A_PASSES; ++p)
            if ((p & 3) == s) MOTE_DMA_A(st_nx2, kt + 2, p);
#pragma unroll
          for (int i = 0; i < W_PER_WAVE; ++i)
            if (((i + 1) & 3) == s) MOTE_DMA_W(st_nx2, kt + 2, i);
        }
        if (s < 3) {
#pragma unroll
          for (int i = 0; i < BM_W; ++i)
            if (!SKIP || i * 32 < rows_w)
              af[(s + 1) & 1][i] = *reinterpret_cast<const v4i*>(st + lds_a_offset(a_row_base + i * 32, 2 * (s + 1) + g));
        }
        if (!SKIP || rows_w > 0) {
#pragma unroll
          for (int m = 0; m < NMAT; ++m)
#pragma unroll
            for (int f = 0; f < BN_W; ++f) {
              const v4i bf = unpack_codes(wf[m][f][s]);
#pragma unroll
              for (int i = 0; i < BM_W; ++i)
                if (!SKIP || i * 32 < rows_w)
                  acc[m][i][f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf, af[s & 1][i], acc[m][i][f], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep each quarter's loads with its quarter
      }
      // K step kt+1 landed everywhere (kt+2 stays in flight); after the last step: every
      // wavefront has read its last stage
      MOTE_WAIT_BARRIER(pf);
      const int t = st_cur; st_cur = st_nxt; st_nxt = st_nx2; st_nx2 = t;
    }

    MOTE_TP(2)
    // (3) start the next tile now: its first two K steps travel while this tile runs its
    // epilogue.  The stage of the last K step (now st_nx2) is free until the next tile's
    // first barrier: it holds the epilogue patches.
    int ktl2 = ktl;
    if (has_next) {
      ktl2 = min(ktp2, KT - kc2 * ktp2);
      MOTE_POINTERS(expert2, nt2, kc2, ktp2);
      MOTE_DMA_META(par ^ 1);
      MOTE_ISSUE_STEP(st_cur, 0);
      if (ktl2 > 1) MOTE_ISSUE_STEP(st_nxt, 1);
    }

    MOTE_TP(3)
    // ---- epilogue ----
    // In registers lane l owns dispatch row r32 and runs of four consecutive output channels
    // (8q + 4g .. +3).  Each wavefront writes one 32-row block of PATCH_F fragments into its
    // private LDS patch and reads it back row-major, 16 bytes per lane, so that a global store
    // instruction covers whole rows of the block.
    constexpr int PATCH_F = Cfg::PATCH_F;
    constexpr int PATCH_ROW = Cfg::PATCH_ROW;
    constexpr int OUT_ROW_BYTES = PATCH_F * 32 * Cfg::OUT_BYTES;
    constexpr int LANES_PER_ROW = OUT_ROW_BYTES / 16;
    constexpr int ROWS_PER_READ = 64 / LANES_PER_ROW;
    static_assert(Cfg::WAVES * Cfg::PATCH_BYTES <= STAGE_BYTES, "the patches fit the free stage");
    if constexpr (Cfg::MODE == 1) {   // a pair cut into K planes: tell the combine kernel how many to add for these rows and channels
      if (planes_t > 1 && kc == 0 && tid < rows) atomicOr(a.plan.row_planes + row0 + tid, (planes_t - 1) << (2 * nt));
    }
    // The lane id is read afresh so that the epilogue's lane-dependent addresses are computed here
    // and not held in registers across the K loop (10-30 registers per configuration).
    int lane_e;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_e));
    const int r32e = lane_e & 31, ge = lane_e >> 5;
    unsigned char* const patch = s_lds + st_nx2 + wave * Cfg::PATCH_BYTES;
    const int rd_row = lane_e / LANES_PER_ROW, rd_chunk = lane_e % LANES_PER_ROW;
#pragma unroll
    for (int i = 0; i < BM_W; ++i) {
      if ((SKIP && i * 32 >= rows_w) || (SKIP_ == 1 && rows_w <= 0)) continue;   // nothing to store
      const int rl = wm * BM_W * 32 + i * 32 + r32e;
      float sg = 0.0f, su = 0.0f;
      if constexpr (Cfg::MODE == 0) {
        const float sx = s_beta[par][rl] / 127.0f;
        sg = sx * al0;
        su = sx * al1;
      }
#pragma unroll
      for (int f0 = 0; f0 < BN_W; f0 += PATCH_F) {
#pragma unroll
        for (int ff = 0; ff < PATCH_F; ++ff) {
          const int f = f0 + ff;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int pcol = ff * 32 + 8 * q + 4 * ge;      // channel inside the patch row
            const int col = f0 * 32 + pcol;                // channel inside the wavefront's block
            if constexpr (Cfg::MODE == 0) {
              float hv[4];
#pragma unroll
              for (int j = 0; j < 4; ++j)
                hv[j] = (static_cast<float>(acc[1][i][f][4 * q + j]) * su) *
                        silu_fast(static_cast<float>(acc[0][i][f][4 * q + j]) * sg);
              uint2 packed;
              packed.x = cvt_pk_bf16(hv[0], hv[1]);
              packed.y = cvt_pk_bf16(hv[2], hv[3]);
              *reinterpret_cast<uint2*>(patch + r32e * PATCH_ROW + pcol * 2) = packed;
              if ((a.tap_gate != nullptr || a.tap_up != nullptr) && rl < rows && n_wave0 + col < N) {   // parity taps (tests only), each optional
                const int64_t o = static_cast<int64_t>(row0 + rl) * N + n_wave0 + col;
                if (a.tap_gate != nullptr)
                  *reinterpret_cast<int4*>(a.tap_gate + o) = make_int4(acc[0][i][f][4 * q], acc[0][i][f][4 * q + 1],
                                                                       acc[0][i][f][4 * q + 2], acc[0][i][f][4 * q + 3]);
                if (a.tap_up != nullptr)
                  *reinterpret_cast<int4*>(a.tap_up + o) = make_int4(acc[1][i][f][4 * q], acc[1][i][f][4 * q + 1],
                                                                     acc[1][i][f][4 * q + 2], acc[1][i][f][4 * q + 3]);
              }
            } else {
              *reinterpret_cast<int4*>(patch + r32e * PATCH_ROW + pcol * 4) = make_int4(
                  acc[0][i][f][4 * q], acc[0][i][f][4 * q + 1], acc[0][i][f][4 * q + 2], acc[0][i][f][4 * q + 3]);
            }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int rd_n = n_wave0 + f0 * 32 + rd_chunk * (16 / Cfg::OUT_BYTES);   // first output channel of this lane's 16 bytes
#pragma unroll
        for (int p = 0; p < 32 / ROWS_PER_READ; ++p) {
          const int pr = p * ROWS_PER_READ + rd_row;
          const u4 v = *reinterpret_cast<const u4*>(patch + pr * PATCH_ROW + rd_chunk * 16);
          const int orow = wm * BM_W * 32 + i * 32 + pr;
          if (orow < rows && rd_n < N) {
            const int64_t o = static_cast<int64_t>(row0 + orow) * N + rd_n;
            if constexpr (Cfg::MODE == 0) *reinterpret_cast<u4*>(a.h + o) = v;
            else *reinterpret_cast<u4*>(a.acc_out + static_cast<int64_t>(kc) * a.partial_stride + o) = v;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
    MOTE_TP(4)
#ifdef MOTE_TRACE
    if (Cfg::MODE == MOTE_TRACE && tid == 0 && tile_it < 32) g_trace[(blockIdx.x * 32 + tile_it) * 8 + 7] = wall_clock64();
    if (Cfg::MODE == MOTE_TRACE && tid == 0 && tile_it < 32) g_trace[(blockIdx.x * 32 + tile_it) * 8 + 5] = (unsigned long long)mt << 32 | (unsigned)nt;
    ++tile_it;
#endif
    if (!has_next) break;
    // Thread 0 draws the ticket of tile i + 2; the others read it after the next tile's first
    // barrier.  The draw is waited for here: the other wavefronts spend that time at the barrier
    // in any case, until the next tile's first K step has landed.
    if (tid == 0) {
      int cur = s_sched[0];
      const int t = next_ticket(cur, tile_i + 2);
      s_sched[0] = cur;
      s_ticket[tile_i & 1] = t;
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    // No barrier here: the patches are private and their stage is not refilled before the next
    // tile's first barrier, the metadata of the next tile went to the other parity buffer.
    par ^= 1;
    ticket = nticket; ++tile_i; mt = mt2; nt = nt2; kc = kc2; expert = expert2; row0 = row02; rows = rows2; ktl = ktl2; ktp_t = ktp2; planes_t = planes2;
  }
#ifdef MOTE_TRACE
  if (Cfg::MODE == MOTE_TRACE && tid == 0 && tile_it < 32) g_trace[(blockIdx.x * 32 + tile_it) * 8 + 4] = 0;
#endif
#undef MOTE_DECODE
#undef MOTE_GATHER
#undef MOTE_POINTERS
#undef MOTE_DMA
#undef MOTE_DMA_A
#undef MOTE_DMA_META
#undef MOTE_DMA_W
#undef MOTE_ISSUE_STEP
#undef MOTE_WAIT_BARRIER
}

#ifdef MOTE_TRACE
extern "C" int mote_debug_trace(void* dst, size_t bytes, int clear) {
  if (clear) { void* p; hipGetSymbolAddress(&p, HIP_SYMBOL(g_trace)); return (int)hipMemset(p, 0, sizeof(g_trace)); }
  return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_trace), bytes);
}
#endif

static int device_cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
  }
  return n;
}

// Workgroups of this configuration that fit on one CU (registers and LDS), from the runtime.
template <typename Cfg>
static int resident_blocks() {
  static int n = 0;
  if (n == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, routed_gemm_kernel<Cfg, 1>, Cfg::THREADS, 0) != hipSuccess || n <= 0)
      n = Cfg::MIN_BLOCKS;
  }
  return n;
}

// Row tiles per band of the tile order (knob group_m; a value
// larger than the number of row tiles gives the plain row-tile-fastest sweep).
int tile_group_m() {
  // default 2; steady state, 2 against 8: T = 2048 at the 3B width 0.464 vs 0.474 ms, C5 11.60 vs 11.65 ms, C2 equal; 1 costs 3 % at the 0.5B width
  const int v = knob(kKnobGroupM);
  return v < 1 ? 2 : v;
}

constexpr int kAllStatic = kFixedShares;   // n_static of a launch that never draws

// Tiles per workgroup from which the tiles are drawn dynamically.
static int routed_dynamic_rounds() {
  const int v = knob(kKnobDynamicRounds);
  return v < 1 ? 1 : v;
}

template <typename Cfg>
static hipError_t launch_cfg(const RoutedGemmArgs& a, int kplanes, hipStream_t stream) {
  const int n_ntiles = (a.N + Cfg::BN - 1) / Cfg::BN;
  const int KT = a.K >> 7;
  const int ktp = (KT + kplanes - 1) / kplanes;
  kplanes = (KT + ktp - 1) / ktp;   // every plane non-empty
  const int64_t tiles = static_cast<int64_t>(a.max_tiles) * n_ntiles * kplanes;
  int64_t blocks = static_cast<int64_t>(device_cu_count()) * resident_blocks<Cfg>();
  if (blocks > tiles) blocks = (tiles + 7) / 8 * 8;
  // tiles drawn from the counters once a workgroup sees several of them, fixed shares otherwise
  // (max_tiles bounds the row tiles for any routing; the expected number is rows / tile_m plus a few)
  const int64_t expected = std::min<int64_t>(a.max_tiles, a.out_rows / a.tile_m + 8) * n_ntiles * kplanes;
  const int n_static = expected >= routed_dynamic_rounds() * blocks ? 1 : kAllStatic;
  // few rows per expert: most row tiles are partly filled (T = 512 at the 3B width with 16 experts:
  // gate-up 88.8 -> 73.2 us, down 47.6 -> 40.1 us; T = 1024: 134 -> 116 us)
  const int64_t n_experts = std::max<int64_t>(1, a.max_tiles - a.out_rows / a.tile_m);
  if (a.out_rows <= 160 * n_experts)
    routed_gemm_kernel<Cfg, 2><<<static_cast<unsigned>(blocks), Cfg::THREADS, 0, stream>>>(a, n_ntiles, kplanes, ktp, tile_group_m(), n_static);
  else
    routed_gemm_kernel<Cfg, 1><<<static_cast<unsigned>(blocks), Cfg::THREADS, 0, stream>>>(a, n_ntiles, kplanes, ktp, tile_group_m(), n_static);
  return hipGetLastError();
}

// Knob routed_variant: selects the tile
// configuration of the large-batch kernels.
static int routed_variant() { return knob(kKnobRoutedVariant); }

// Plan tile height by the average number of rows an expert sees: 32-row tiles for few rows
// (decode kernels), 64-row tiles for some tens of rows where the wave-streaming kernel fits the
// shape (the weights are then streamed once per 64 rows; the large-batch kernel would run half-empty
// 128-row tiles and re-read the activations for every channel tile), else 128.
int routed_tile_m(int T, int k, int E, int d, int F) {
  const int64_t avg = (static_cast<int64_t>(T) * k + E - 1) / E;
  if (avg > knob(kKnobMidRowsLo) && avg <= knob(kKnobMidRowsHi) && routed_mid_kernel_fits(d, F)) return 64;
  if (avg <= 48) return 32;
  return 128;
}

hipError_t launch_routed_gate_up(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  switch (routed_variant()) {
    case 1: return launch_cfg<RoutedCfg<0, 4, 1, 1, 4, 2>>(a, 1, stream);   // 4 wavefronts of 128 x (32+32)
    case 2: return launch_cfg<RoutedCfg<0, 2, 2, 2, 2, 2>>(a, 1, stream);   // 4 wavefronts of 64 x (64+64)
    default: return launch_cfg<RoutedCfg<0, 2, 1, 2, 4, 4>>(a, 1, stream);  // 8 wavefronts of 64 x (32+32): four per SIMD (2-3 % faster)
  }
}

// K planes of the large-batch down projection (see shared_down_planes): pure function of the
// shape, the number of row tiles is estimated as R/128 + E/2.
int routed_down_planes(int T, int k, int E, int d, int F) {
  const int64_t mtiles = (static_cast<int64_t>(T) * k) / 128 + (E + 1) / 2;
  const int64_t tiles = mtiles * ((d + 127) / 128);
  const int KT = F >> 7;
  int planes = tiles > 0 ? static_cast<int>((512 + tiles / 2) / tiles) : 1;
  // between one and two workgroups per CU's worth of 128 x 128 tiles, two planes of 128-wide tiles fill the
  // chip better than one plane of 256-wide ones (3B width, 16 experts: T = 1024 398 -> 367 us per forward,
  // T = 1536 520 -> 503 us; from T = 2048 on, 640 tiles, no gain, and a loss at T = 3072)
  if (planes == 1 && tiles < knob(kKnobDownSplitTiles)) planes = 2;
  if (planes > F / 2048) planes = F / 2048;   // every plane adds an int32 partial output (C2, F = 4864: 2 planes 30 us, 3 planes 41 us)
  int fill = tiles > 0 ? static_cast<int>(256 / tiles) : 1;   // few tiles: up to one workgroup per CU, planes of at least 4 K steps
  if (fill > KT / 4) fill = KT / 4;
  if (planes < fill) planes = fill;
  if (planes > 8) planes = 8;
  if (planes < 1) planes = 1;
  const int ktp = (KT + planes - 1) / planes;
  return (KT + ktp - 1) / ktp;
}

static int routed_down_variant() {
  const int v = knob(kKnobRoutedDownVariant);
  return v < 0 ? routed_variant() : v;
}

// Channels per tile of the large-batch down projection (the unit of plan.row_planes).
int routed_down_tile_n(int planes) {
  if (planes > 1) return RoutedCfg<1, 2, 2, 2, 2, 2>::BN;
  switch (routed_down_variant()) {
    case 1: return RoutedCfg<1, 4, 2, 1, 4, 2>::BN;
    case 2: return RoutedCfg<1, 2, 2, 2, 2, 2>::BN;
    default: return RoutedCfg<1, 2, 4, 2, 2, 2>::BN;
  }
}

hipError_t launch_routed_down(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  if (a.planes > 1) return launch_cfg<RoutedCfg<1, 2, 2, 2, 2, 2>>(a, a.planes, stream);   // small problem: 128 x 128 tiles
  switch (routed_down_variant()) {
    case 1: return launch_cfg<RoutedCfg<1, 4, 2, 1, 4, 2>>(a, 1, stream);
    case 2: return launch_cfg<RoutedCfg<1, 2, 2, 2, 2, 2>>(a, 1, stream);
    default: return launch_cfg<RoutedCfg<1, 2, 4, 2, 2, 2>>(a, 1, stream);
  }
}

}  // namespace mote
