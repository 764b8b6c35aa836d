// Grouped ternary GEMMs of the routed experts (Eq.5-6, and the ternary linear layer
// Y = Q_w(W) Q_a(x) at the end of Section 3.1) on int8 MFMA with int32 accumulation.
//
//   gate-up mode : G = t_gate . q_x, U = t_up . q_x for the rows of one expert, then the
//                  fused epilogue  h = bf16( (U*s_u) * SiLU(G*s_g) ),  s = beta_x/127 * alpha
//   down mode    : D = t_down . q_h, stored as int32 (the combine kernel applies the scales)
//
// Work decomposition: the dispatch plan lists row tiles (one expert each, BM rows); a
// workgroup owns one row tile x one block of BN output channels and walks K in steps of
// 128.  Activations (int8, gathered through tok_of in gate-up mode) are staged in LDS,
// 16-byte chunks XOR-swizzled by row so that ds_read_b128 of 32 consecutive rows is
// conflict free.  Packed weights never touch LDS: a tile of 32 rows x 128 channels is
// 1 KiB = one 16-byte load per lane, each 32-bit word expands with (w >> 2j) & 0x03030303
// into the four operand registers of one v_mfma_i32_32x32x32_i8.  The codes are t+1, so
// the accumulator holds sum (t+1) q; the row sum of q is subtracted in the epilogue.
//
// MFMA operand mapping (32x32x32 i8): first operand = weights, lane l supplies output
// channel l%32 and 16 consecutive input channels of half l/32; second operand =
// activations, lane l supplies dispatch row l%32 and the same 16 channels.  Result register
// v of lane l is output channel 8*(v/4) + 4*(l/32) + v%4 of dispatch row l%32.
//
// Epilogue: every wavefront transposes its result fragments through a private LDS patch so
// that the global stores are whole rows of 128 (bf16) or 256 (int32) contiguous bytes.
#include <stdlib.h>

#include "common.h"
#include "launch.h"

namespace mote {

template <int MODE_, int BM_W_, int BN_W_, int WAVES_M_, int WAVES_N_, int MIN_BLOCKS_ = 1>
struct RoutedCfg {
  static constexpr int MODE = MODE_;  // 0 gate-up (two matrices, SwiGLU epilogue), 1 down
  static constexpr int NMAT = MODE_ == 0 ? 2 : 1;
  static constexpr int BM_W = BM_W_, BN_W = BN_W_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int MIN_BLOCKS = MIN_BLOCKS_;  // workgroups per CU the register budget must allow
  static constexpr int BM = 32 * BM_W_ * WAVES_M_;
  static constexpr int BN = 32 * BN_W_ * WAVES_N_;
  static constexpr int WAVES = WAVES_M_ * WAVES_N_;
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int ROWS_PER_PASS = THREADS / 8;
  static constexpr int A_PASSES = BM / ROWS_PER_PASS;
  static constexpr int STAGE_BYTES = BM * 128;
  // epilogue patch of one wavefront: 32 rows x (BN_W*32 outputs) + 16 bytes of row padding
  static constexpr int OUT_BYTES = MODE_ == 0 ? 2 : 4;
  static constexpr int PATCH_ROW = BN_W_ * 32 * OUT_BYTES + 16;
  static constexpr int PATCH_BYTES = 32 * PATCH_ROW;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES > WAVES * PATCH_BYTES ? 2 * STAGE_BYTES : WAVES * PATCH_BYTES;
  static_assert(BM % ROWS_PER_PASS == 0, "activation loader covers the tile in whole passes");
  static_assert(64 % (BN_W_ * 32 * OUT_BYTES / 16) == 0, "an epilogue read covers whole rows");
};

__device__ __forceinline__ v4i unpack_codes(uint32_t w) {
  v4i b;
  b.x = static_cast<int>(w & 0x03030303u);
  b.y = static_cast<int>((w >> 2) & 0x03030303u);
  b.z = static_cast<int>((w >> 4) & 0x03030303u);
  b.w = static_cast<int>((w >> 6) & 0x03030303u);
  return b;
}

// LDS tile geometry: 128-byte rows of eight 16-byte chunks, chunk index XOR-swizzled with
// bits 1..3 of the row.  Two consecutive rows span the 64 banks once, so 16 lanes that read
// the same chunk of 16 consecutive rows (one quarter of a ds_read_b128) hit 16 distinct
// 4-bank groups: conflict free (measured 2x faster than swizzling with row bits 0..2).
__device__ __forceinline__ int lds_a_offset(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

// One 128-channel K step of a wavefront is four 32-channel sub-steps; each reads BM_W
// activation fragments from LDS and, per weight fragment, unpacks 16 codes per lane and feeds
// BM_W MFMAs (MOTE_KSTEP in the kernel).  The global loads of the NEXT K step are spread over
// the four sub-steps: issued in one burst right after the barrier, eight wavefronts x eight
// 1-KiB loads fill the CU's vector-memory queue and every wavefront stalls in issue (measured:
// about 800 cycles per K step) before it reaches its first MFMA.
template <typename Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_BLOCKS) void routed_gemm_kernel(RoutedGemmArgs a, int n_ntiles, int kplanes, int ktp) {
  constexpr int NMAT = Cfg::NMAT, BM_W = Cfg::BM_W, BN_W = Cfg::BN_W;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, THREADS = Cfg::THREADS;
  static_assert(BM <= THREADS, "one thread per tile row publishes the row metadata");
  __shared__ __attribute__((aligned(16))) unsigned char s_a[Cfg::LDS_BYTES];
  __shared__ float s_scale[BM];
  __shared__ int s_rs[BM];

  const int K = a.K, N = a.N;
  const int KT = K >> 7;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int wn_u = __builtin_amdgcn_readfirstlane(wn);   // wavefront-uniform: keeps weight bases scalar
  const int r32 = lane & 31, g = lane >> 5;
  const int a_row_base = wm * BM_W * 32 + r32;
  const unsigned char* const q_base = reinterpret_cast<const unsigned char*>(a.q);
  const int64_t expert_words = static_cast<int64_t>(N) * K / 16;
  unsigned char* const stage0 = s_a;
  unsigned char* const stage1 = s_a + Cfg::STAGE_BYTES;

  // Persistent workgroups: the grid is one wave of resident workgroups; each walks a strided
  // list of (row tile, channel tile) pairs.  Workgroups are dealt to the 8 XCDs round-robin
  // by linear id, so XCD x takes the channel tiles x, x+8, ... (or, when there are fewer
  // than 16 channel tiles, the row tiles x, x+8, ...) and walks the other index fastest:
  // the packed weights of an expert and the few activation row tiles in flight stay
  // resident in that XCD's own L2.
  // With kplanes > 1 (down projection of small problems) the contraction is cut into planes
  // of ktp K steps; a (channel tile, plane) pair then plays the role of a channel tile and each
  // plane writes its own partial output that the combine kernel adds.
  n_ntiles *= kplanes;
  const int xcd = blockIdx.x & 7;
  const int n_mtiles = a.plan.n_tiles[0];
  const bool split_n = n_ntiles >= 16;
  const int xcd_ntiles = split_n ? (n_ntiles - xcd + 7) >> 3 : n_ntiles;
  const int xcd_mtiles = split_n ? n_mtiles : (n_mtiles - xcd + 7) >> 3;
  const int xcd_work = xcd_ntiles * xcd_mtiles;
  const int stride = gridDim.x >> 3;
  int slot = blockIdx.x >> 3;
  if (slot >= xcd_work) return;

  // Loader state of the tile being contracted.  The same variables are refilled for the
  // NEXT tile while the current one is still in its epilogue (see the end of the loop).
  // Addresses are kept as uniform 64-bit bases (scalar registers) plus 32-bit per-lane byte
  // offsets, so each global load needs one address VGPR.
  uint32_t a_off[Cfg::A_PASSES];           // byte offset of this thread's row chunk inside q
  int a_dst[Cfg::A_PASSES];
  const unsigned char* w_base[NMAT][BN_W]; // uniform: first packed tile of the fragment's channel rows
  const uint32_t w_lane = lane * 16;
  u4 w_a[NMAT][BN_W], w_b[NMAT][BN_W];
  u4 a_reg[Cfg::A_PASSES];
  int src_row[Cfg::A_PASSES];   // row of q (gathered) per loader pass
  int meta_row = 0;             // row whose beta / rowsum this thread publishes (tid < BM)
  float meta_beta = 1.0f;
  int meta_rs = 0;
  int mt, nt, kc, expert, row0, rows;
#pragma unroll
  for (int p = 0; p < Cfg::A_PASSES; ++p) a_dst[p] = lds_a_offset(p * Cfg::ROWS_PER_PASS + (tid >> 3), tid & 7);

#define MOTE_DECODE(slot_, mt_, nt_, kc_)                                       \
  {                                                                             \
    const int mi_ = (slot_) / xcd_ntiles, ni_ = (slot_) - mi_ * xcd_ntiles;     \
    mt_ = split_n ? mi_ : xcd + 8 * mi_;                                        \
    const int ntk_ = split_n ? xcd + 8 * ni_ : ni_;                             \
    nt_ = ntk_ / kplanes;                                                       \
    kc_ = ntk_ - nt_ * kplanes;                                                 \
  }
#define MOTE_GATHER(row0_, rows_)                                                                  \
  {                                                                                                \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p) {                                    \
      const int rslot_ = (row0_) + min(p * Cfg::ROWS_PER_PASS + (tid >> 3), (rows_)-1);            \
      src_row[p] = a.gather ? a.gather[rslot_] : rslot_;                                           \
    }                                                                                              \
    const int mslot_ = (row0_) + min(tid < BM ? tid : 0, (rows_)-1);                               \
    meta_row = a.gather ? a.gather[mslot_] : mslot_;                                               \
  }
#define MOTE_POINTERS(expert_, nt_, kc_)                                                           \
  {                                                                                                \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                                      \
      a_off[p] = static_cast<uint32_t>(src_row[p]) * static_cast<uint32_t>(K) + (tid & 7) * 16 +   \
                 static_cast<uint32_t>((kc_) * ktp) * 128u;                                        \
    _Pragma("unroll") for (int f = 0; f < BN_W; ++f) {                                             \
      const int n_frag_ = (nt_) * BN + wn_u * BN_W * 32 + f * 32;                                  \
      const int nt32_ = (n_frag_ < N ? n_frag_ : 0) >> 5; /* fragments past N read tile 0 */       \
      const int64_t off_ = (static_cast<int64_t>(expert_) * expert_words +                         \
                            (static_cast<int64_t>(nt32_) * KT + (kc_) * ktp) * 256) * 4;           \
      w_base[0][f] = reinterpret_cast<const unsigned char*>(a.w_gate) + off_;                      \
      if constexpr (NMAT == 2) w_base[1][f] = reinterpret_cast<const unsigned char*>(a.w_up) + off_; \
    }                                                                                              \
    meta_beta = a.beta[meta_row];                                                                  \
    meta_rs = a.rowsum[meta_row];                                                                  \
  }
#define MOTE_LOAD_W(dst_, kt_)                                                  \
  _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                              \
    _Pragma("unroll") for (int f = 0; f < BN_W; ++f)                            \
      dst_[m][f] = *reinterpret_cast<const u4*>(w_base[m][f] + static_cast<int64_t>(kt_) * 1024 + w_lane)
#define MOTE_LOAD_A(kt_)                                                        \
  _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                     \
    a_reg[p] = *reinterpret_cast<const u4*>(q_base + static_cast<int64_t>(kt_) * 128 + a_off[p])
#define MOTE_STORE_A(stage_)                                                    \
  _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                     \
    *reinterpret_cast<u4*>((stage_) + a_dst[p]) = a_reg[p]

  // ---- first tile: the whole dependent chain (plan -> gather -> rows) is paid once ----
  MOTE_DECODE(slot, mt, nt, kc);
  expert = a.plan.tile_expert[mt];
  row0 = a.plan.tile_row0[mt];
  rows = a.plan.tile_rows[mt];
  MOTE_GATHER(row0, rows);
  MOTE_POINTERS(expert, nt, kc);
  MOTE_LOAD_A(0);
  MOTE_LOAD_W(w_a, 0);

  for (;;) {
    // (1) publish this tile's row metadata and first activation K step
    if (tid < BM) {
      s_scale[tid] = meta_beta / 127.0f;
      s_rs[tid] = meta_rs;
    }
    MOTE_STORE_A(stage0);
    // (2) coordinates of the next tile of this workgroup (uniform scalar loads)
    const int nslot = slot + stride;
    const bool has_next = nslot < xcd_work;
    int mt2 = mt, nt2 = nt, kc2 = kc, expert2 = expert, row02 = row0, rows2 = rows;
    if (has_next) {
      MOTE_DECODE(nslot, mt2, nt2, kc2);
      expert2 = a.plan.tile_expert[mt2];
      row02 = a.plan.tile_row0[mt2];
      rows2 = a.plan.tile_rows[mt2];
    }
    __syncthreads();
    const int n_wave0 = nt * BN + wn * BN_W * 32;  // first output channel of this wavefront

    // Accumulators start at -rowsum(q): the stored codes are t+1, so sum (t+1) q - sum q = sum t q.
    v16i acc[NMAT][BM_W][BN_W];
#pragma unroll
    for (int i = 0; i < BM_W; ++i) {
      const int nrs = kc == 0 ? -s_rs[wm * BM_W * 32 + i * 32 + r32] : 0;   // the correction enters plane 0 only
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < BN_W; ++f)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[m][i][f][v] = nrs;
    }

    // (3) K loop.  Unrolled by two K steps so that the two weight register sets and the two
    // LDS stages are named statically (no register copies on the back-edge): while K step kt
    // is contracted, the packed weights and the activation tile of kt+1 are in flight.
    const int ktl = min(ktp, KT - kc * ktp);   // K steps of this plane
    // Quarter in which each load of the next K step is issued.  Gate-up: one activation pass and one
    // weight fragment per quarter; down: the activation passes first (their LDS store comes first).
#define MOTE_PF_A(p) (Cfg::MODE == 0 ? ((p) & 3) : 0)
#define MOTE_PF_W(j) ((j) & 3)
#define MOTE_KSTEP(stage_, wc_, wn_, ktn_, PREFETCH_)                                                   \
  {                                                                                                    \
    v4i af_[2][BM_W];                                                                                  \
    _Pragma("unroll") for (int i = 0; i < BM_W; ++i)                                                   \
      af_[0][i] = *reinterpret_cast<const v4i*>((stage_) + lds_a_offset(a_row_base + i * 32, g));      \
    _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                                    \
      if (PREFETCH_) { /* quarter s of the next K step's loads */                                      \
        _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                                      \
          if (MOTE_PF_A(p) == s) a_reg[p] = *reinterpret_cast<const u4*>(q_base + static_cast<int64_t>(ktn_) * 128 + a_off[p]); \
        _Pragma("unroll") for (int j = 0; j < NMAT * BN_W; ++j)                                        \
          if (MOTE_PF_W(j) == s) wn_[j / BN_W][j % BN_W] = *reinterpret_cast<const u4*>(                    \
              w_base[j / BN_W][j % BN_W] + static_cast<int64_t>(ktn_) * 1024 + w_lane);                \
      }                                                                                                \
      if (s < 3) {                                                                                     \
        _Pragma("unroll") for (int i = 0; i < BM_W; ++i)                                               \
          af_[(s + 1) & 1][i] = *reinterpret_cast<const v4i*>((stage_) + lds_a_offset(a_row_base + i * 32, 2 * (s + 1) + g)); \
      }                                                                                                \
      _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                                 \
        _Pragma("unroll") for (int f = 0; f < BN_W; ++f) {                                             \
          const v4i bf_ = unpack_codes(wc_[m][f][s]);                                                  \
          _Pragma("unroll") for (int i = 0; i < BM_W; ++i)                                             \
            acc[m][i][f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf_, af_[s & 1][i], acc[m][i][f], 0, 0, 0); \
        }                                                                                              \
      __builtin_amdgcn_sched_barrier(0);  /* keep each quarter's loads with its quarter */             \
    }                                                                                                  \
  }
    int kt = 0;
    for (; kt + 1 < ktl; kt += 2) {
      MOTE_KSTEP(stage0, w_a, w_b, kt + 1, true);
      MOTE_STORE_A(stage1);
      __syncthreads();
      const int kn = min(kt + 2, ktl - 1);  // the last prefetch of an even-length loop is a harmless repeat
      MOTE_KSTEP(stage1, w_b, w_a, kn, true);
      MOTE_STORE_A(stage0);
      __syncthreads();
    }
    if (kt < ktl) MOTE_KSTEP(stage0, w_a, w_b, 0, false);
#undef MOTE_KSTEP
#undef MOTE_PF_A
#undef MOTE_PF_W

    // (4) start the next tile now: its gather indices, row scalars and first K step travel
    // while this tile runs its epilogue.
    if (has_next) {
      MOTE_GATHER(row02, rows2);
      MOTE_POINTERS(expert2, nt2, kc2);
      MOTE_LOAD_A(0);
      MOTE_LOAD_W(w_a, 0);
    }
    __syncthreads();  // every wavefront is done with the activation stages: LDS becomes epilogue space

    // ---- epilogue ----
    // In registers lane l owns dispatch row r32 and runs of four consecutive output channels
    // (8q + 4g .. +3).  Each wavefront writes one 32-row fragment row into its LDS patch and
    // reads it back row-major, 16 bytes per lane, so every global store covers whole rows.
    constexpr int PATCH_ROW = Cfg::PATCH_ROW;
    constexpr int OUT_ROW_BYTES = BN_W * 32 * Cfg::OUT_BYTES;   // 128 (bf16) or 256 (int32) for BN_W = 2
    constexpr int LANES_PER_ROW = OUT_ROW_BYTES / 16;
    constexpr int ROWS_PER_READ = 64 / LANES_PER_ROW;
    unsigned char* const patch = s_a + wave * Cfg::PATCH_BYTES;
    const float al0 = a.alpha[expert * 3 + (Cfg::MODE == 0 ? 0 : 2)];
    const float al1 = Cfg::MODE == 0 ? a.alpha[expert * 3 + 1] : 0.0f;
    const int rd_row = lane / LANES_PER_ROW, rd_chunk = lane % LANES_PER_ROW;
    const int rd_n = n_wave0 + rd_chunk * (16 / Cfg::OUT_BYTES);   // first output channel of this lane's 16 bytes
#pragma unroll
    for (int i = 0; i < BM_W; ++i) {
      const int rl = wm * BM_W * 32 + i * 32 + r32;
      float sg = 0.0f, su = 0.0f;
      if constexpr (Cfg::MODE == 0) {
        const float sx = s_scale[rl];
        sg = sx * al0;
        su = sx * al1;
      }
#pragma unroll
      for (int f = 0; f < BN_W; ++f) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = f * 32 + 8 * q + 4 * g;
          if constexpr (Cfg::MODE == 0) {
            float hv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
              hv[j] = (static_cast<float>(acc[1][i][f][4 * q + j]) * su) *
                      silu_fast(static_cast<float>(acc[0][i][f][4 * q + j]) * sg);
            uint2 packed;
            packed.x = cvt_pk_bf16(hv[0], hv[1]);
            packed.y = cvt_pk_bf16(hv[2], hv[3]);
            *reinterpret_cast<uint2*>(patch + r32 * PATCH_ROW + col * 2) = packed;
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
            *reinterpret_cast<int4*>(patch + r32 * PATCH_ROW + col * 4) = make_int4(
                acc[0][i][f][4 * q], acc[0][i][f][4 * q + 1], acc[0][i][f][4 * q + 2], acc[0][i][f][4 * q + 3]);
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
    if (!has_next) break;
    __syncthreads();  // LDS (patches, row metadata) is reused by the next tile
    slot = nslot; mt = mt2; nt = nt2; kc = kc2; expert = expert2; row0 = row02; rows = rows2;
  }
#undef MOTE_DECODE
#undef MOTE_GATHER
#undef MOTE_POINTERS
#undef MOTE_LOAD_W
#undef MOTE_LOAD_A
#undef MOTE_STORE_A
}

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
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, routed_gemm_kernel<Cfg>, Cfg::THREADS, 0) != hipSuccess || n <= 0)
      n = Cfg::MIN_BLOCKS;
  }
  return n;
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
  routed_gemm_kernel<Cfg><<<static_cast<unsigned>(blocks), Cfg::THREADS, 0, stream>>>(a, n_ntiles, kplanes, ktp);
  return hipGetLastError();
}

// Tuning switch (environment variable MOTE_ROUTED_VARIANT, read once): selects the tile
// configuration of the large-batch kernels.
static int routed_variant() {
  static int v = -1;
  if (v < 0) {
    const char* e = getenv("MOTE_ROUTED_VARIANT");
    v = e ? atoi(e) : 0;
  }
  return v;
}

// Plan tile height: 32-row tiles when experts see few rows (decode), else 128.
int routed_tile_m(int T, int k, int E) {
  const int64_t avg = (static_cast<int64_t>(T) * k + E - 1) / E;
  if (avg <= 48) return 32;
  return 128;
}

hipError_t launch_routed_gate_up(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  switch (routed_variant()) {
    case 1: return launch_cfg<RoutedCfg<0, 4, 1, 1, 4, 2>>(a, 1, stream);
    default: return launch_cfg<RoutedCfg<0, 2, 2, 2, 2, 2>>(a, 1, stream);
  }
}

// K planes of the large-batch down projection (see shared_down_planes): pure function of the
// shape, the number of row tiles is estimated as R/128 + E/2.
int routed_down_planes(int T, int k, int E, int d, int F) {
  const int64_t mtiles = (static_cast<int64_t>(T) * k) / 128 + (E + 1) / 2;
  const int64_t tiles = mtiles * ((d + 127) / 128);
  const int KT = F >> 7;
  int planes = static_cast<int>(512 / (tiles > 0 ? tiles : 1));
  if (planes > 8) planes = 8;
  if (planes > KT / 4) planes = KT / 4;
  if (planes < 1) planes = 1;
  const int ktp = (KT + planes - 1) / planes;
  return (KT + ktp - 1) / ktp;
}

hipError_t launch_routed_down(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  if (a.planes > 1) return launch_cfg<RoutedCfg<1, 2, 2, 2, 2, 2>>(a, a.planes, stream);   // small problem: 128 x 128 tiles
  switch (routed_variant()) {
    case 1: return launch_cfg<RoutedCfg<1, 4, 2, 1, 4, 2>>(a, 1, stream);
    case 2: return launch_cfg<RoutedCfg<1, 2, 2, 2, 2, 2>>(a, 1, stream);
    default: return launch_cfg<RoutedCfg<1, 2, 4, 2, 2, 2>>(a, 1, stream);
  }
}

}  // namespace mote
