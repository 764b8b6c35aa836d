// Shared expert FFN(x) of Eq.2: the dense checkpoint's full-precision SwiGLU FFN, active
// for every token.  bf16 operands on v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
//   gate-up mode : g = x W_gate^T, u = x W_up^T, h_s = bf16(u * SiLU(g))     [T, F]
//   down mode    : y_s = h_s W_down^T (fp32)                                 [T, d]
//
// Both operands are K-contiguous ([rows, K] row-major) and are loaded straight into LDS
// (buffer_load ... lds, 16 bytes per lane) in K steps of 32 elements: a tile row is 64
// bytes = four 16-byte chunks, chunk index XOR-swizzled with bits 2..3 of the row so that a
// ds_read_b128 of 16 consecutive rows touches every LDS bank once.  Three stages, requested
// two K steps ahead; two workgroups of four wavefronts share a CU, so the epilogue and the
// barrier waits of one overlap with the MFMAs of the other.  Persistent workgroups walk an
// XCD-aware list of (row tile, channel tile, K plane) triples as the ternary GEMM does.
//
// MFMA operand mapping (32x32x16 bf16): first operand = weights (lane l: output channel
// l%32, 8 consecutive K elements of half l/32), second = activations (lane l: token row
// l%32); result register v of lane l is output channel 8*(v/4) + 4*(l/32) + v%4 of token
// row l%32.
#include <stdlib.h>

#include "common.h"
#include "launch.h"

namespace mote {

template <int MODE_, int BM_W_, int BN_W_, int WAVES_M_, int WAVES_N_, int MIN_BLOCKS_ = 1, int STAGES_ = 3>
struct SharedCfg {
  static constexpr int MIN_BLOCKS = MIN_BLOCKS_;
  static constexpr int STAGES = STAGES_;   // LDS ring: 3, or 4 with the fragment reads of a K step moved half a step ahead
  static constexpr int MODE = MODE_;  // 0 gate-up (two matrices, SwiGLU epilogue), 1 down
  static constexpr int NMAT = MODE_ == 0 ? 2 : 1;
  static constexpr int BM_W = BM_W_, BN_W = BN_W_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int BM = 32 * BM_W_ * WAVES_M_;
  static constexpr int BN = 32 * BN_W_ * WAVES_N_;   // output channels per matrix
  static constexpr int WAVES = WAVES_M_ * WAVES_N_;
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int KSTEP = 32;                   // bf16 elements per K step: 64-byte tile rows
  static constexpr int ROWS_PER_PASS = 16 * WAVES;   // a wavefront load fills 16 tile rows
  static constexpr int A_PASSES = BM / ROWS_PER_PASS;
  static constexpr int B_PASSES = NMAT * BN / ROWS_PER_PASS;
  static constexpr int A_BYTES = BM * 64;
  static constexpr int B_BYTES = BN * 64;            // per matrix
  static constexpr int STAGE_BYTES = A_BYTES + NMAT * B_BYTES;
  static constexpr int OUT_BYTES = MODE_ == 0 ? 2 : 4;
  static constexpr int PATCH_F = MODE_ == 0 ? BN_W_ : 1;   // fragments per epilogue pass (128-byte output rows for 2 / 1)
  static constexpr int PATCH_ROW = PATCH_F * 32 * OUT_BYTES + 16;
  static constexpr int PATCH_BYTES = 32 * PATCH_ROW;
  static constexpr bool PATCH_IN_STAGE = WAVES * PATCH_BYTES <= STAGE_BYTES;
  // ring of four: two stages are free during the epilogue, each takes the patches of half the wavefronts
  static constexpr bool PATCH_IN_TWO = STAGES_ == 4 && (WAVES / 2) * PATCH_BYTES <= STAGE_BYTES;
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + ((PATCH_IN_STAGE || PATCH_IN_TWO) ? 0 : WAVES * PATCH_BYTES);
  static_assert(STAGES == 3 || STAGES == 4, "ring of three or four stages");
  static_assert(STAGES == 3 || PATCH_IN_TWO, "the ring of four keeps the epilogue patches in its two free stages");
  static_assert(BM % ROWS_PER_PASS == 0 && (NMAT * BN) % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0,
                "loaders cover the tiles in whole passes, a pass stays inside one matrix");
  static_assert(64 % (PATCH_F * 32 * OUT_BYTES / 16) == 0, "an epilogue read covers whole rows");
  static_assert(A_PASSES + B_PASSES < 16, "fits the low vmcnt field");
};

// 64-byte rows of four 16-byte chunks, chunk XOR-swizzled with row bits 2..3: the 16 lanes of
// a quarter wavefront read one chunk of 16 consecutive rows = all 64 banks exactly once.
__device__ __forceinline__ int lds_tile_offset(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4); }

struct SharedGemmArgs {
  const uint16_t* act;   // [M, K] bf16
  const uint16_t* w0;    // [N, K] bf16 (gate / down)
  const uint16_t* w1;    // [N, K] bf16 (up)
  int M, N, K;
  uint16_t* h_out;       // gate-up: bf16 [M, N]
  float* y_out;          // down: fp32 [planes][M, N]
  int64_t plane_stride;  // elements between partial planes
  const float* scale0;   // optional fp32 [N]: the sums of w0 (w1) are multiplied by scale0 (scale1)
  const float* scale1;   // per output channel (RTN-quantised weights held as integer-valued bf16)
};

// Grouped rows: group e owns the rows row0[e] .. row0[e+1]-1 of act / the output and the row tiles
// tile0[e] .. tile0[e+1]-1 (ceil(rows / BM) of them, none for an empty group); its weights are matrix e
// of w0 ([n][N, K]) and its channel scales row e of scale0 ([n][N]).  A row tile that reaches beyond its
// group's last row loads the rows that follow (clamped to the last row of act) and stores only its own.
constexpr int kMaxRowGroups = 64;
struct RowGroups {
  int n;
  int row0[kMaxRowGroups + 1];
  int tile0[kMaxRowGroups + 1];
};

// GROUPED: 0 plain, 1 row groups (above), 2 K ranges: plane p of the kplanes = rg->n planes contracts the
// K range row0[p] .. row0[p+1]-1 (multiples of 64 elements; an empty range gives a plane of zeros).
template <typename Cfg, int GROUPED>
__device__ __forceinline__ void shared_gemm_body(const SharedGemmArgs& a, const RowGroups* rg, int n_ntiles, int kplanes,
                                                 int ktp, int group_m) {
  constexpr int NMAT = Cfg::NMAT, BM_W = Cfg::BM_W, BN_W = Cfg::BN_W;
  constexpr int BM = Cfg::BM, BN = Cfg::BN;
  constexpr int A_BYTES = Cfg::A_BYTES, B_BYTES = Cfg::B_BYTES, STAGE_BYTES = Cfg::STAGE_BYTES;
  constexpr int NLOAD = Cfg::A_PASSES + Cfg::B_PASSES;   // vector-memory operations a wavefront issues per K step
  extern __shared__ __attribute__((aligned(16))) unsigned char s_lds[];

  const int M = a.M, N = a.N, K = a.K;
  const int KT = K >> 5;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int r32 = lane & 31, g = lane >> 5;
  const int a_row_base = wm * BM_W * 32 + r32;
  const int b_row_base = wn * BN_W * 32 + r32;
  // LDS byte address of the stage area (what M0 takes for a direct-to-LDS load)
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)s_lds);

  // Persistent workgroups, dealt to the 8 XCDs round-robin by linear id: XCD x owns the
  // (channel tile, K plane) pairs x, x+8, ... (the row tiles x, x+8, ... when there are fewer
  // than 16 pairs); inside an XCD the tiles are ordered in bands of group_m row tiles, row tile
  // fastest, so the resident workgroups share both activation tiles and weight slices in L2.
  // With kplanes > 1 (down projection of small problems) the contraction is cut into planes of
  // ktp K steps; each plane writes its own partial output, added later in plane order.
  n_ntiles *= kplanes;
  int n_mtiles = (M + BM - 1) / BM;
  if constexpr (GROUPED == 1) n_mtiles = rg->tile0[rg->n];
  const int xcd = blockIdx.x & 7;
  const bool split_n = n_ntiles >= 16;
  const int xcd_ntiles = split_n ? (n_ntiles - xcd + 7) >> 3 : n_ntiles;
  const int xcd_mtiles = split_n ? n_mtiles : (n_mtiles - xcd + 7) >> 3;
  const int xcd_work = xcd_ntiles * xcd_mtiles;
  const int per_group = group_m * xcd_ntiles;   // tiles of a band of group_m row tiles
  const int stride = gridDim.x >> 3;
  int slot = blockIdx.x >> 3;
  if (slot >= xcd_work) return;

  // Loader: raw buffer loads written in assembly (the compiler has no exact model of
  // outstanding direct-to-LDS loads across this loop).  Vector-memory operations complete in
  // issue order, so waiting for "all but the NLOAD youngest" retires the K step that is about
  // to be contracted while the following one stays in flight; anything else issued since
  // (stores of the previous epilogue) only makes that wait stricter.
  constexpr int kBufferFlags = 0x00020000;   // raw buffer, 32-bit data format
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
  const v4i rsrc_b0 = make_rsrc(a.w0, static_cast<int64_t>(GROUPED == 1 ? rg->n : 1) * N * K * 2);
  const v4i rsrc_b1 = make_rsrc(NMAT == 2 ? a.w1 : a.w0, static_cast<int64_t>(N) * K * 2);
  // lane l of a wavefront load lands at byte 16*l of a 1-KiB block = tile row l/4, physical
  // chunk l%4, and therefore fetches logical chunk (l%4) ^ swizzle(row)
  const int ld_row = wave_u * 16 + (lane >> 2);
  const uint32_t ld_chunk = static_cast<uint32_t>(((lane & 3) ^ ((lane >> 4) & 3)) << 4);
  uint32_t a_off[Cfg::A_PASSES], b_off[Cfg::B_PASSES];   // byte offsets of this lane's 16 bytes, K step 0 of the plane
  int mt, nt, kc, ktl;
  // first row of the tile, one past the last row it may store, its group (0 without groups)
  int mrow, mend = M, grp = 0;
  int st_cur = 0, st_nxt = STAGE_BYTES, st_nx2 = 2 * STAGE_BYTES;   // stage of K step kt, kt+1, kt+2 (byte offsets)
  int st_nx3 = 3 * STAGE_BYTES;                                      // ... and kt+3 (ring of four stages only)

#define MOTE_DECODE(slot_, mt_, nt_, kc_)                                       \
  {                                                                             \
    const int grp_ = (slot_) / per_group;                                       \
    const int in_ = (slot_) - grp_ * per_group;                                 \
    const int gsz_ = min(xcd_mtiles - grp_ * group_m, group_m);                 \
    const int ni_ = in_ / gsz_, mi_ = grp_ * group_m + (in_ - ni_ * gsz_);      \
    mt_ = split_n ? mi_ : xcd + 8 * mi_;                                        \
    const int ntk_ = split_n ? xcd + 8 * ni_ : ni_;                             \
    nt_ = ntk_ / kplanes;                                                       \
    kc_ = ntk_ - nt_ * kplanes;                                                 \
  }
  // where row tile mt_ starts and ends (uniform; the group is found by walking the table)
#define MOTE_ROWS(mt_, mrow_, mend_, grp_)                                      \
  {                                                                             \
    if constexpr (GROUPED == 1) {                                               \
      int e_ = 0;                                                               \
      while (e_ + 1 < rg->n && rg->tile0[e_ + 1] <= (mt_)) ++e_;                \
      grp_ = e_;                                                                \
      mrow_ = rg->row0[e_] + ((mt_) - rg->tile0[e_]) * BM;                      \
      mend_ = rg->row0[e_ + 1];                                                 \
    } else {                                                                    \
      mrow_ = (mt_) * BM;                                                       \
    }                                                                           \
  }
  // byte offset of plane kc_ in an operand row and its K steps (uniform; GROUPED == 2 reads them from the
  // table, early enough that the scalar loads are back when the tile starts)
#define MOTE_KRANGE(kc_, kb_, ktl_)                                                                \
  {                                                                                                \
    if constexpr (GROUPED == 2) {                                                                  \
      kb_ = static_cast<uint32_t>(rg->row0[kc_]) * 2u;                                             \
      ktl_ = (rg->row0[(kc_) + 1] - rg->row0[kc_]) >> 5;                                           \
    } else {                                                                                       \
      kb_ = static_cast<uint32_t>((kc_) * ktp) * 64u;                                              \
      ktl_ = min(ktp, KT - (kc_) * ktp);                                                           \
    }                                                                                              \
  }
#define MOTE_POINTERS(mrow_, grp_, nt_, kb_)                                                       \
  {                                                                                                \
    const uint32_t k0_ = (kb_) + ld_chunk;                                                         \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p) {                                    \
      const int row_ = min((mrow_) + p * Cfg::ROWS_PER_PASS + ld_row, M - 1);                      \
      a_off[p] = static_cast<uint32_t>(row_) * static_cast<uint32_t>(K) * 2u + k0_;                \
    }                                                                                              \
    _Pragma("unroll") for (int p = 0; p < Cfg::B_PASSES; ++p) {                                    \
      const int row_ = min((nt_) * BN + (p * Cfg::ROWS_PER_PASS) % BN + ld_row, N - 1) + (grp_) * N; \
      b_off[p] = static_cast<uint32_t>(row_) * static_cast<uint32_t>(K) * 2u + k0_;                \
    }                                                                                              \
  }
  // one 16-byte-per-lane direct load: LDS byte address (uniform), lane offset, buffer, scalar offset
#define MOTE_DMA(lds_, voff_, rsrc_, soff_)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"           \
               :: "s"(lds_), "v"(voff_), "s"(rsrc_), "s"(soff_) : "memory")
#define MOTE_DMA_A(stage_, ks_, p_)                                                                \
  MOTE_DMA(lds0 + (stage_) + ((p_) * Cfg::ROWS_PER_PASS + wave_u * 16) * 64, a_off[p_], rsrc_a, (ks_) * 64)
  // loader pass p_ of the weights: matrix (p_*ROWS_PER_PASS)/BN, rows (p_*ROWS_PER_PASS)%BN ... of it
#define MOTE_DMA_B(stage_, ks_, p_)                                                                \
  MOTE_DMA(lds0 + (stage_) + A_BYTES + ((p_) * Cfg::ROWS_PER_PASS + wave_u * 16) * 64, b_off[p_],  \
           (((p_) * Cfg::ROWS_PER_PASS) / BN == 0 ? rsrc_b0 : rsrc_b1), (ks_) * 64)
#define MOTE_ISSUE_STEP(stage_, ks_)                                                               \
  {                                                                                                \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p) MOTE_DMA_A(stage_, ks_, p);          \
    _Pragma("unroll") for (int p = 0; p < Cfg::B_PASSES; ++p) MOTE_DMA_B(stage_, ks_, p);          \
  }
  // in_flight_: whether the loads of one more K step were issued after the ones needed now
#define MOTE_WAIT_BARRIER(in_flight_)                                                              \
  {                                                                                                \
    if (in_flight_) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NLOAD) : "memory");                  \
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                          \
    asm volatile("s_barrier" ::: "memory");                                                        \
  }

  // ---- first tile ----
  MOTE_DECODE(slot, mt, nt, kc);
  MOTE_ROWS(mt, mrow, mend, grp);
  uint32_t kb;
  MOTE_KRANGE(kc, kb, ktl);
  MOTE_POINTERS(mrow, grp, nt, kb);
  MOTE_ISSUE_STEP(st_cur, 0);
  if (ktl > 1) MOTE_ISSUE_STEP(st_nxt, 1);

  for (;;) {
    const int nslot = slot + stride;
    const bool has_next = nslot < xcd_work;
    int mt2 = mt, nt2 = nt, kc2 = kc;
    int mrow2 = mrow, mend2 = mend, grp2 = grp, ktl2 = ktl;
    uint32_t kb2 = kb;
    if (has_next) {
      MOTE_DECODE(nslot, mt2, nt2, kc2);
      MOTE_ROWS(mt2, mrow2, mend2, grp2);
      MOTE_KRANGE(kc2, kb2, ktl2);
    }
    MOTE_WAIT_BARRIER(ktl > 1);   // K step 0 visible to every wavefront; the patches of the previous tile are done
    if constexpr (Cfg::STAGES == 4) {   // the third K step goes where patches of the previous tile were
      if (ktl > 2) MOTE_ISSUE_STEP(st_nx2, 2);
    }

    v16f acc[NMAT][BM_W][BN_W];
#pragma unroll
    for (int m = 0; m < NMAT; ++m)
#pragma unroll
      for (int i = 0; i < BM_W; ++i)
#pragma unroll
        for (int f = 0; f < BN_W; ++f)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[m][i][f][v] = 0.0f;

    if constexpr (Cfg::STAGES == 4) {
      // Ring of four stages, loads three K steps ahead, ONE barrier per K step placed in the middle
      // of the step: after it the next step's stage is visible, and its first-half fragments are
      // read while the MFMAs of this step's second half run; the second-half fragments of a step
      // are read at its start, under the MFMAs of the first half.  The wavefronts of the single
      // workgroup of a CU all stop at the same barrier, so without this every K step began with
      // the matrix pipe idle for an LDS round trip.
      constexpr int NH0 = (Cfg::A_PASSES + 1) / 2 + (Cfg::B_PASSES + 1) / 2;   // loads issued in the first half of a step
      bf16x8 af0[BM_W], bf0[NMAT][BN_W], af1[BM_W], bf1[NMAT][BN_W];
#define MOTE_READ_HALF(af_, bf_, stage_, s_)                                                              \
      {                                                                                                   \
        const unsigned char* const st_ = s_lds + (stage_);                                                \
        _Pragma("unroll") for (int i = 0; i < BM_W; ++i)                                                  \
          af_[i] = *reinterpret_cast<const bf16x8*>(st_ + lds_tile_offset(a_row_base + i * 32, 2 * (s_) + g)); \
        _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                                  \
          _Pragma("unroll") for (int f = 0; f < BN_W; ++f)                                                \
            bf_[m][f] = *reinterpret_cast<const bf16x8*>(st_ + A_BYTES + m * B_BYTES +                    \
                                                         lds_tile_offset(b_row_base + f * 32, 2 * (s_) + g)); \
      }
      // One half of a K step: the MFMAs of fragments (ua_, ub_), and between them - so that the matrix
      // pipe never waits for this wavefront to get through a block of other instructions - the reads of
      // the next half's fragments (fa_, fb_) from (fstage_, sub-step fs_), two per MFMA, then the
      // direct loads of parity par_ of K step ks_ into dstage_, one per MFMA.  Every wavefront of the
      // workgroup is in the same half at the same time, so nothing else would cover such a block.
      constexpr int NM = NMAT * BN_W * BM_W;          // MFMAs of a half
      constexpr int NR = BM_W + NMAT * BN_W;          // fragment reads of a half
      constexpr int RPS = 2;                          // fragment reads per MFMA (1: C3 shared down 5 % slower, 3: the same)
      constexpr int RSLOTS = (NR + RPS - 1) / RPS;
#define MOTE_SIDE_READ(r_, fa_, fb_, fstage_, fs_)                                                        \
      if ((r_) < BM_W) {                                                                                  \
        fa_[(r_) < BM_W ? (r_) : 0] = *reinterpret_cast<const bf16x8*>(                                   \
            s_lds + (fstage_) + lds_tile_offset(a_row_base + ((r_) < BM_W ? (r_) : 0) * 32, 2 * (fs_) + g)); \
      } else if ((r_) < NR) {                                                                             \
        const int b_ = (r_) < NR && (r_) >= BM_W ? (r_) - BM_W : 0;                                       \
        fb_[b_ / BN_W][b_ % BN_W] = *reinterpret_cast<const bf16x8*>(                                     \
            s_lds + (fstage_) + A_BYTES + (b_ / BN_W) * B_BYTES + lds_tile_offset(b_row_base + (b_ % BN_W) * 32, 2 * (fs_) + g)); \
      }
      // the d_-th direct load of parity par_: the A passes par_, par_ + 2, ..., then the B passes
#define MOTE_SIDE_DMA(d_, par_, dstage_, ks_)                                                             \
      {                                                                                                   \
        constexpr int NA_ = (Cfg::A_PASSES - (par_) + 1) / 2, NB_ = (Cfg::B_PASSES - (par_) + 1) / 2;     \
        if ((d_) >= 0 && (d_) < NA_) { MOTE_DMA_A(dstage_, ks_, ((d_) >= 0 && (d_) < NA_ ? 2 * (d_) + (par_) : 0)); } \
        else if ((d_) >= NA_ && (d_) < NA_ + NB_) { MOTE_DMA_B(dstage_, ks_, ((d_) >= NA_ && (d_) < NA_ + NB_ ? 2 * ((d_) - NA_) + (par_) : 0)); } \
      }
#define MOTE_HALF(ua_, ub_, fill_, fa_, fb_, fstage_, fs_, dma_, par_, dstage_, ks_)                      \
      {                                                                                                   \
        _Pragma("unroll") for (int m_ = 0; m_ < NMAT; ++m_)                                               \
          _Pragma("unroll") for (int f_ = 0; f_ < BN_W; ++f_)                                             \
            _Pragma("unroll") for (int i_ = 0; i_ < BM_W; ++i_) {                                         \
              const int j_ = (m_ * BN_W + f_) * BM_W + i_;                                                \
              acc[m_][i_][f_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ub_[m_][f_], ua_[i_], acc[m_][i_][f_], 0, 0, 0); \
              if (fill_) {                                                                                \
                _Pragma("unroll") for (int r_ = 0; r_ < RPS; ++r_)                                        \
                  MOTE_SIDE_READ(RPS * j_ + r_, fa_, fb_, fstage_, fs_)                                   \
              }                                                                                           \
              if (dma_) MOTE_SIDE_DMA(j_ - RSLOTS, par_, dstage_, ks_)                                    \
              __builtin_amdgcn_sched_barrier(0);                                                          \
            }                                                                                             \
        /* more side work than MFMAs (small tiles): the rest at the end */                                \
        _Pragma("unroll") for (int j_ = NM; j_ < RSLOTS + (Cfg::A_PASSES + Cfg::B_PASSES + 1) / 2; ++j_) { \
          if (fill_) {                                                                                    \
            _Pragma("unroll") for (int r_ = 0; r_ < RPS; ++r_)                                            \
              MOTE_SIDE_READ(RPS * j_ + r_, fa_, fb_, fstage_, fs_)                                       \
          }                                                                                               \
          if (dma_) MOTE_SIDE_DMA(j_ - RSLOTS, par_, dstage_, ks_)                                        \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
      }
      MOTE_READ_HALF(af0, bf0, st_cur, 0);
      for (int kt = 0; kt < ktl; ++kt) {
        const bool pf = kt + 3 < ktl;
        __builtin_amdgcn_sched_barrier(0);
        // first half: fragments of sub-step 1 of this step; first half of the loads of K step kt+3,
        // into the stage that step kt-1 used
        MOTE_HALF(af0, bf0, true, af1, bf1, st_cur, 1, pf, 0, st_nx3, kt + 3)
        // K step kt+1 has landed everywhere (kt+2 and the half of kt+3 stay in flight); every
        // wavefront has finished its reads of this step's stage
        if (pf) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(NLOAD + NH0) : "memory");
        else if (kt + 2 < ktl) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(NLOAD) : "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
        // second half: fragments of sub-step 0 of the next step (after the last step: of a stage nobody
        // uses, read and dropped); the other half of the loads
        MOTE_HALF(af1, bf1, true, af0, bf0, st_nxt, 0, pf, 1, st_nx3, kt + 3)
        const int t = st_cur; st_cur = st_nxt; st_nxt = st_nx2; st_nx2 = st_nx3; st_nx3 = t;
      }
#undef MOTE_HALF
#undef MOTE_SIDE_DMA
#undef MOTE_SIDE_READ
#undef MOTE_READ_HALF
    } else {
      // K loop.  K step kt contracts stage st_cur while the loads of kt+2 are issued, half of them
      // per 16-element sub-step, into the stage that the barrier at the end of step kt-1 released.
      for (int kt = 0; kt < ktl; ++kt) {
        const bool pf = kt + 2 < ktl;
        const unsigned char* const st = s_lds + st_cur;
        // all fragments of the step are requested at once: the MFMAs of the first half run while
        // those of the second half are still on their way
        bf16x8 af[2][BM_W], bfr[2][NMAT][BN_W];
  #pragma unroll
        for (int s = 0; s < 2; ++s) {
  #pragma unroll
          for (int i = 0; i < BM_W; ++i)
            af[s][i] = *reinterpret_cast<const bf16x8*>(st + lds_tile_offset(a_row_base + i * 32, 2 * s + g));
  #pragma unroll
          for (int m = 0; m < NMAT; ++m)
  #pragma unroll
            for (int f = 0; f < BN_W; ++f)
              bfr[s][m][f] = *reinterpret_cast<const bf16x8*>(st + A_BYTES + m * B_BYTES +
                                                              lds_tile_offset(b_row_base + f * 32, 2 * s + g));
        }
        __builtin_amdgcn_sched_barrier(0);
  #pragma unroll
        for (int s = 0; s < 2; ++s) {
          if (pf) {   // half s of the loads of K step kt+2
  #pragma unroll
            for (int p = 0; p < Cfg::A_PASSES; ++p)
              if ((p & 1) == s) MOTE_DMA_A(st_nx2, kt + 2, p);
  #pragma unroll
            for (int p = 0; p < Cfg::B_PASSES; ++p)
              if ((p & 1) == s) MOTE_DMA_B(st_nx2, kt + 2, p);
          }
  #pragma unroll
          for (int m = 0; m < NMAT; ++m)
  #pragma unroll
            for (int f = 0; f < BN_W; ++f)
  #pragma unroll
              for (int i = 0; i < BM_W; ++i)
                acc[m][i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s][m][f], af[s][i], acc[m][i][f], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);  // keep each half's loads with its half
        }
        // K step kt+1 landed everywhere (kt+2 stays in flight); after the last step: every
        // wavefront has read its last stage
        MOTE_WAIT_BARRIER(pf);
        const int t = st_cur; st_cur = st_nxt; st_nxt = st_nx2; st_nx2 = t;
      }
    }

    // Start the next tile now: its first two K steps travel while this tile runs its epilogue.
    // The stage of the last K step (now st_nx2) is free until the next tile's first barrier.
    if (has_next) {
      MOTE_POINTERS(mrow2, grp2, nt2, kb2);
      MOTE_ISSUE_STEP(st_cur, 0);
      if (ktl2 > 1) MOTE_ISSUE_STEP(st_nxt, 1);
    }

    // ---- epilogue ----
    // In registers lane l owns token row r32 and runs of four consecutive output channels
    // (8q + 4g .. +3).  Each wavefront writes one 32-row block of PATCH_F fragments into its
    // private LDS patch and reads it back row-major, 16 bytes per lane, so that a global store
    // instruction covers whole 128-byte rows of the block.
    constexpr int PATCH_F = Cfg::PATCH_F;
    constexpr int PATCH_ROW = Cfg::PATCH_ROW;
    constexpr int OUT_ROW_BYTES = PATCH_F * 32 * Cfg::OUT_BYTES;
    constexpr int LANES_PER_ROW = OUT_ROW_BYTES / 16;
    constexpr int ROWS_PER_READ = 64 / LANES_PER_ROW;
    unsigned char* const patch =
        Cfg::PATCH_IN_TWO ? s_lds + (wave < Cfg::WAVES / 2 ? st_nx2 : st_nx3) + (wave % (Cfg::WAVES / 2)) * Cfg::PATCH_BYTES
                          : s_lds + (Cfg::PATCH_IN_STAGE ? st_nx2 : Cfg::STAGES * STAGE_BYTES) + wave * Cfg::PATCH_BYTES;
    const int m0 = mrow, n_wave0 = nt * BN + wn * BN_W * 32;
    const int rd_row = lane / LANES_PER_ROW, rd_chunk = lane % LANES_PER_ROW;
    if (a.scale0 != nullptr) {   // row scales of quantised weights (uniform branch, not taken by the bf16 expert)
#pragma unroll
      for (int f = 0; f < BN_W; ++f) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ch = min(n_wave0 + f * 32 + 8 * q + 4 * g, N - 4);
          const float4 s0 = *reinterpret_cast<const float4*>(a.scale0 + static_cast<int64_t>(grp) * N + ch);
          float4 s1 = s0;
          if constexpr (NMAT == 2) s1 = *reinterpret_cast<const float4*>(a.scale1 + ch);
#pragma unroll
          for (int i = 0; i < BM_W; ++i) {
            acc[0][i][f][4 * q] *= s0.x; acc[0][i][f][4 * q + 1] *= s0.y; acc[0][i][f][4 * q + 2] *= s0.z; acc[0][i][f][4 * q + 3] *= s0.w;
            if constexpr (NMAT == 2) {
              acc[1][i][f][4 * q] *= s1.x; acc[1][i][f][4 * q + 1] *= s1.y; acc[1][i][f][4 * q + 2] *= s1.z; acc[1][i][f][4 * q + 3] *= s1.w;
            }
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < BM_W; ++i) {
#pragma unroll
      for (int f0 = 0; f0 < BN_W; f0 += PATCH_F) {
#pragma unroll
        for (int ff = 0; ff < PATCH_F; ++ff) {
          const int f = f0 + ff;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int pcol = ff * 32 + 8 * q + 4 * g;   // channel inside the patch row
            if constexpr (Cfg::MODE == 0) {
              float hv[4];
#pragma unroll
              for (int j = 0; j < 4; ++j) hv[j] = acc[NMAT - 1][i][f][4 * q + j] * silu_fast(acc[0][i][f][4 * q + j]);
              uint2 packed;
              packed.x = cvt_pk_bf16(hv[0], hv[1]);
              packed.y = cvt_pk_bf16(hv[2], hv[3]);
              *reinterpret_cast<uint2*>(patch + r32 * PATCH_ROW + pcol * 2) = packed;
            } else {
              *reinterpret_cast<float4*>(patch + r32 * PATCH_ROW + pcol * 4) = make_float4(
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
          const int orow = m0 + wm * BM_W * 32 + i * 32 + pr;
          if (orow < mend && rd_n < N) {
            const int64_t o = static_cast<int64_t>(orow) * N + rd_n;
            if constexpr (Cfg::MODE == 0) *reinterpret_cast<u4*>(a.h_out + o) = v;
            else *reinterpret_cast<u4*>(a.y_out + static_cast<int64_t>(kc) * a.plane_stride + o) = v;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
    if (!has_next) break;
    // No barrier here: the patches are private and their stage is not refilled before the next
    // tile's first barrier.
    slot = nslot; mt = mt2; nt = nt2; kc = kc2; ktl = ktl2;
    mrow = mrow2; mend = mend2; grp = grp2; kb = kb2;
  }
#undef MOTE_DECODE
#undef MOTE_ROWS
#undef MOTE_KRANGE
#undef MOTE_POINTERS
#undef MOTE_DMA
#undef MOTE_DMA_A
#undef MOTE_DMA_B
#undef MOTE_ISSUE_STEP
#undef MOTE_WAIT_BARRIER
}

template <typename Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_BLOCKS) void shared_gemm_kernel(SharedGemmArgs a, int n_ntiles,
                                                                                   int kplanes, int ktp, int group_m) {
  shared_gemm_body<Cfg, 0>(a, nullptr, n_ntiles, kplanes, ktp, group_m);
}

template <typename Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_BLOCKS) void grouped_gemm_kernel(SharedGemmArgs a, RowGroups rg,
                                                                                    int n_ntiles, int kplanes, int ktp,
                                                                                    int group_m) {
  shared_gemm_body<Cfg, 1>(a, &rg, n_ntiles, kplanes, ktp, group_m);
}

template <typename Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_BLOCKS) void kgrouped_gemm_kernel(SharedGemmArgs a, RowGroups rg,
                                                                                     int n_ntiles, int group_m) {
  shared_gemm_body<Cfg, 2>(a, &rg, n_ntiles, rg.n, 0, group_m);
}

static int shared_cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
  }
  return n;
}

static int shared_variant() { return knob(kKnobSharedVariant); }

// kplanes64 / the plane length are counted in 64-element units (the workspace layout depends
// on shared_down_planes, which predates the 32-element K step).
template <typename Cfg>
static hipError_t launch_shared_cfg(const SharedGemmArgs& a, int kplanes, hipStream_t stream) {
  const int n_ntiles = (a.N + Cfg::BN - 1) / Cfg::BN;
  const int KT64 = a.K >> 6;
  const int ktp = 2 * ((KT64 + kplanes - 1) / kplanes);   // K steps of 32 per plane
  const int n_mtiles = (a.M + Cfg::BM - 1) / Cfg::BM;
  const size_t lds = Cfg::LDS_BYTES;
  static bool attr_set = false;
  static int resident = Cfg::MIN_BLOCKS;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(shared_gemm_kernel<Cfg>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, shared_gemm_kernel<Cfg>, Cfg::THREADS, lds) == hipSuccess && n > 0)
      resident = n;
    attr_set = true;
  }
  const int64_t tiles = static_cast<int64_t>(n_mtiles) * n_ntiles * kplanes;
  int64_t blocks = static_cast<int64_t>(shared_cu_count()) * resident;
  if (blocks > tiles) blocks = (tiles + 7) / 8 * 8;
  shared_gemm_kernel<Cfg><<<static_cast<unsigned>(blocks), Cfg::THREADS, lds, stream>>>(a, n_ntiles, kplanes, ktp, tile_group_m());
  return hipGetLastError();
}

hipError_t launch_shared_gate_up(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up, int T, int d,
                                 int F, uint16_t* h_s, hipStream_t stream) {
  return launch_shared_gate_up_scaled(x, w_gate, w_up, nullptr, nullptr, T, d, F, h_s, stream);
}

hipError_t launch_shared_gate_up_scaled(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up,
                                        const float* s_gate, const float* s_up, int T, int d, int F, uint16_t* h_s,
                                        hipStream_t stream) {
  if (T == 0) return hipSuccess;
  SharedGemmArgs a{x, w_gate, w_up, T, F, d, h_s, nullptr, 0, s_gate, s_up};
  // Operand traffic per flop halves with a 256 x 256 tile (one 8-wavefront workgroup per CU): the
  // 128-row tile at two workgroups per CU saturates the L2 -> L1 path first.  Small problems keep
  // the 128-row tile, which leaves fewer CUs idle in the last round.  Of its two forms, eight
  // wavefronts of 64 x (32+32) are faster alone (C2: 47.8 vs 49.7 us) but fill every wavefront
  // slot of a CU; four wavefronts of 64 x (64+64) leave room for the routed chain's kernels that
  // run beside it, and the whole forward is faster (C2 steady state: 0.1563 vs 0.1643 ms).
  int v = shared_variant();
  if (v == 0) v = static_cast<int64_t>((T + 255) / 256) * ((F + 127) / 128) >= 384 ? 5 : 3;
  // fewer 128 x (128+128) tiles than fill the workgroup slots: half-width tiles (d=896, T=512:
  // 0.090 -> 0.083 ms per forward; d=1536, T=512: 0.143 -> 0.131 ms).  Not below four row tiles:
  // at most one full-width tile per CU then, and a tile of either width takes about as long
  // (this kernel alone, T=256: d=896 14.7 vs 18.7 us, d=1536 24 vs 38 us, d=2048 31 vs 49 us).
  if (shared_variant() == 0 && (T + 127) / 128 >= 4 &&
      static_cast<int64_t>((T + 127) / 128) * ((F + 127) / 128) < 300)
    v = 1;
  switch (v) {
    case 1: return launch_shared_cfg<SharedCfg<0, 2, 1, 2, 2, 2>>(a, 1, stream);   // 128 x (64+64)
    case 2: return launch_shared_cfg<SharedCfg<0, 2, 2, 4, 2, 1>>(a, 1, stream);   // 256 x (128+128), 8 wavefronts, 1 workgroup / CU
    case 5: return launch_shared_cfg<SharedCfg<0, 2, 2, 4, 2, 1, 4>>(a, 1, stream);   // the same with the ring of four stages (C5 4.08 -> 4.02 ms)
    case 4: return launch_shared_cfg<SharedCfg<0, 2, 1, 2, 4, 4>>(a, 1, stream);   // 128 x (128+128), 8 wavefronts of 64 x (32+32), 2 workgroups / CU
    default: return launch_shared_cfg<SharedCfg<0, 2, 2, 2, 2, 2>>(a, 1, stream);  // 128 x (128+128), 2 workgroups / CU
  }
}

// K planes of the large-batch down projection: enough (row tile, channel tile, plane) triples
// for two workgroups per CU, but planes of at least 2048 channels: every further plane adds an
// fp32 partial output that is written here and read by the combine (C2, F = 4864: four planes
// 42 us, two planes 35 us and a faster combine; the 3B width with T = 2048, F = 11008: one plane
// on 128 of 512 workgroup slots 220 us).  Pure function of the shape: the workspace layout
// depends on it.
// Mid-size batches at the 3B width: 48 to 64 output tiles of 256 x 256, so that four or five K planes
// of them fill the chip once (one workgroup per CU); the big tile moves less operand data per flop
// than two planes of 128 x 128 tiles.  Measured alone this kernel takes 111 -> 84 us at the 3B width with
// T = 2048 (122 -> 87 us on the slower kind of box); the forward, where it shares the chip with the routed
// chain, gains 1 to 3.5 % at T = 2048 and 0 to 2 % at T = 1536.
// Not elsewhere: eight planes at T = 1024 make the combine and the kernels after it slower (371 -> 373 us),
// the 1.5B width (six channel tiles) 293 -> 294 us, the 0.5B width 152 -> 160 us.
static int shared_down_big_planes(int T, int d, int F) {
  const int64_t tiles256 = static_cast<int64_t>((T + 255) / 256) * ((d + 255) / 256);
  if (T < 1536 || d < 2048 || tiles256 > 64) return 0;
  int planes = static_cast<int>(256 / tiles256);
  if (planes > F / 1024) planes = F / 1024;
  return planes >= 2 ? planes : 0;
}

int shared_down_planes(int T, int d, int F) {
  if (const int big = shared_down_big_planes(T, d, F)) {
    const int KT = F >> 6, ktp = (KT + big - 1) / big;
    return (KT + ktp - 1) / ktp;
  }
  const int64_t tiles = static_cast<int64_t>((T + 127) / 128) * ((d + 127) / 128);
  const int KT = F >> 6;
  int planes = tiles > 0 ? static_cast<int>(512 / tiles) : 1;   // rounded down: a third plane at the 1.5B width (192 tiles) cost 5 %
  if (planes > F / 2048) planes = F / 2048;
  // few tiles (small T): the partial outputs are small then, and an empty CU costs more than a
  // plane; up to one workgroup per CU, planes of at least 8 K steps of 64
  int fill = tiles > 0 ? static_cast<int>(256 / tiles) : 1;
  if (fill > KT / 8) fill = KT / 8;
  if (planes < fill) planes = fill;
  if (planes > 8) planes = 8;
  if (planes < 1) planes = 1;
  const int ktp = (KT + planes - 1) / planes;
  return (KT + ktp - 1) / ktp;
}

hipError_t launch_shared_down(const uint16_t* h_s, const uint16_t* w_down, int T, int d, int F, float* y_s,
                              hipStream_t stream) {
  return launch_shared_down_scaled(h_s, w_down, nullptr, T, d, F, y_s, stream);
}

hipError_t launch_shared_down_scaled(const uint16_t* h_s, const uint16_t* w_down, const float* s_down, int T, int d,
                                     int F, float* y_s, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  SharedGemmArgs a{h_s, w_down, nullptr, T, d, F, nullptr, y_s, static_cast<int64_t>(T) * d, s_down, nullptr};
  const int planes = shared_down_planes(T, d, F);
  if (shared_down_big_planes(T, d, F) != 0) return launch_shared_cfg<SharedCfg<1, 2, 4, 4, 2, 1, 4>>(a, planes, stream);
  if (planes > 1) return launch_shared_cfg<SharedCfg<1, 2, 2, 2, 2, 2>>(a, planes, stream);   // small problem: 128 x 128 tiles
  int v = shared_variant();
  if (v == 0) v = static_cast<int64_t>((T + 255) / 256) * ((d + 255) / 256) >= 256 ? 5 : 3;
  switch (v) {
    case 1: return launch_shared_cfg<SharedCfg<1, 2, 2, 2, 2, 2>>(a, 1, stream);    // 128 x 128
    case 2: return launch_shared_cfg<SharedCfg<1, 2, 4, 4, 2, 1>>(a, 1, stream);    // 256 x 256, 8 wavefronts, 1 workgroup / CU
    case 5: return launch_shared_cfg<SharedCfg<1, 2, 4, 4, 2, 1, 4>>(a, 1, stream);    // the same with the ring of four stages (C5 2.15 -> 2.09 ms)
    default: return launch_shared_cfg<SharedCfg<1, 2, 4, 2, 2, 2>>(a, 1, stream);   // 128 x 256
  }
}

template <typename Cfg>
static hipError_t launch_grouped_cfg(const SharedGemmArgs& a, const int32_t* row0, int n_groups, int kplanes,
                                     hipStream_t stream) {
  RowGroups rg;
  rg.n = n_groups;
  int tiles_m = 0;
  for (int e = 0; e < n_groups; ++e) {
    rg.row0[e] = row0[e] - row0[0];
    rg.tile0[e] = tiles_m;
    tiles_m += (row0[e + 1] - row0[e] + Cfg::BM - 1) / Cfg::BM;
  }
  rg.row0[n_groups] = row0[n_groups] - row0[0];
  rg.tile0[n_groups] = tiles_m;
  for (int e = n_groups + 1; e <= kMaxRowGroups; ++e) rg.row0[e] = rg.tile0[e] = 0;
  if (tiles_m == 0) return hipSuccess;
  const int n_ntiles = (a.N + Cfg::BN - 1) / Cfg::BN;
  const int KT64 = a.K >> 6;
  const int ktp = 2 * ((KT64 + kplanes - 1) / kplanes);
  const size_t lds = Cfg::LDS_BYTES;
  static bool attr_set = false;
  static int resident = Cfg::MIN_BLOCKS;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_gemm_kernel<Cfg>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, grouped_gemm_kernel<Cfg>, Cfg::THREADS, lds) == hipSuccess && n > 0)
      resident = n;
    attr_set = true;
  }
  const int64_t tiles = static_cast<int64_t>(tiles_m) * n_ntiles * kplanes;
  int64_t blocks = static_cast<int64_t>(shared_cu_count()) * resident;
  if (blocks > tiles) blocks = (tiles + 7) / 8 * 8;
  grouped_gemm_kernel<Cfg><<<static_cast<unsigned>(blocks), Cfg::THREADS, lds, stream>>>(a, rg, n_ntiles, kplanes, ktp,
                                                                                        tile_group_m());
  return hipGetLastError();
}

// Row tiles a grouped launch has with tiles of bm rows.
static int64_t grouped_row_tiles(const int32_t* row0, int n_groups, int bm) {
  int64_t t = 0;
  for (int e = 0; e < n_groups; ++e) t += (row0[e + 1] - row0[e] + bm - 1) / bm;
  return t;
}

// K planes of a grouped GEMM (pure function of the group sizes and the shape, at most max_planes).  256 x 256
// tiles: two planes when one plane leaves more than 15 % of the last round of workgroups empty and two
// leave less (16 groups of about 1024 rows, N = 2048, K = 11008: 576 tiles on 256 CUs; one / two / three /
// four planes 2.39 / 2.32 / 2.37 / 2.35 ms for the whole backward call), else one.  Small problems
// (128 x 128 tiles): as many as give two workgroups per CU, planes of at least 16 K steps of 64.
int grouped_gemm_planes(const int32_t* row0_host, int n_groups, int N, int K, int max_planes) {
  const int cus = shared_cu_count();
  const int64_t t256 = grouped_row_tiles(row0_host, n_groups, 256) * ((N + 255) / 256);
  if (t256 >= (3 * cus) / 4) {
    auto eff = [&](int p) {
      const int64_t rounds = (t256 * p + cus - 1) / cus;
      return static_cast<double>(t256 * p) / static_cast<double>(rounds * cus);
    };
    if (eff(1) >= 0.85 || max_planes < 2 || (K >> 6) < 32) return 1;
    return eff(2) > eff(1) + 0.05 ? 2 : 1;
  }
  const int64_t t128 = grouped_row_tiles(row0_host, n_groups, 128) * ((N + 127) / 128);
  if (t128 == 0) return 1;
  int planes = static_cast<int>((2 * cus) / t128);
  if (planes > (K >> 6) / 16) planes = (K >> 6) / 16;
  if (planes > max_planes) planes = max_planes;
  return planes < 1 ? 1 : planes;
}

// Grouped GEMM for other callers: rows row0_host[e] .. row0_host[e+1]-1 of act (row0_host: n_groups + 1
// ascending HOST integers; act, out and the rows are counted from row0_host[0], which act and out point at)
// are contracted with matrix e of w ([n_groups][N, K] bf16) and scaled per channel by row e of scale
// ([n_groups][N], optional): out[r, n] = scale[e][n] * sum_k act[r, k] * w[e][n, k].  planes as given by
// grouped_gemm_planes: plane p writes its partial sums to out + p * rows * N and the caller adds them.
// n_groups <= 64, n_groups * N * K * 2 bytes and rows * K * 2 bytes below 4 GiB, K a multiple of 64.
hipError_t launch_gemm_grouped_f32(const uint16_t* act, const uint16_t* w, const int32_t* row0_host, int n_groups, int N,
                                   int K, float* out, const float* scale, int planes, hipStream_t stream) {
  if (n_groups < 1 || n_groups > kMaxRowGroups) return hipErrorInvalidValue;
  const int M = row0_host[n_groups] - row0_host[0];
  if (M == 0 || N == 0) return hipSuccess;
  SharedGemmArgs a{act, w, nullptr, M, N, K, nullptr, out, static_cast<int64_t>(M) * N, scale, nullptr};
  if (grouped_row_tiles(row0_host, n_groups, 256) * ((N + 255) / 256) >= (3 * shared_cu_count()) / 4)
    return launch_grouped_cfg<SharedCfg<1, 2, 4, 4, 2, 1, 4>>(a, row0_host, n_groups, planes, stream);   // 256 x 256
  return launch_grouped_cfg<SharedCfg<1, 2, 2, 2, 2, 2>>(a, row0_host, n_groups, planes, stream);        // 128 x 128
}

template <typename Cfg>
static hipError_t launch_kgrouped_cfg(const SharedGemmArgs& a, const int32_t* k0, int n_groups, hipStream_t stream) {
  RowGroups rg;
  rg.n = n_groups;
  for (int e = 0; e <= kMaxRowGroups; ++e) {
    rg.row0[e] = k0[std::min(e, n_groups)];
    rg.tile0[e] = 0;
  }
  const int n_ntiles = (a.N + Cfg::BN - 1) / Cfg::BN;
  const int n_mtiles = (a.M + Cfg::BM - 1) / Cfg::BM;
  const size_t lds = Cfg::LDS_BYTES;
  static bool attr_set = false;
  static int resident = Cfg::MIN_BLOCKS;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kgrouped_gemm_kernel<Cfg>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kgrouped_gemm_kernel<Cfg>, Cfg::THREADS, lds) == hipSuccess && n > 0)
      resident = n;
    attr_set = true;
  }
  const int64_t tiles = static_cast<int64_t>(n_mtiles) * n_ntiles * n_groups;
  int64_t blocks = static_cast<int64_t>(shared_cu_count()) * resident;
  if (blocks > tiles) blocks = (tiles + 7) / 8 * 8;
  kgrouped_gemm_kernel<Cfg><<<static_cast<unsigned>(blocks), Cfg::THREADS, lds, stream>>>(a, rg, n_ntiles, tile_group_m());
  return hipGetLastError();
}

// Several contractions over consecutive K ranges of the same two operands in one launch: plane p,
// written to out + p * M * N, is sum over k0_host[p] <= k < k0_host[p+1] of act[m, k] * w[n, k] (operands
// [M, K] and [N, K] with K = k0_host[n_groups]; the offsets are HOST integers, multiples of 64, ascending from
// 0; an empty range gives zeros).  The caller's use: one problem per range, its operands side by side along K.
hipError_t launch_gemm_tn_f32_kgroups(const uint16_t* act, const uint16_t* w, int M, int N, const int32_t* k0_host,
                                      int n_groups, float* out, hipStream_t stream) {
  if (n_groups < 1 || n_groups > kMaxRowGroups) return hipErrorInvalidValue;
  if (M == 0 || N == 0) return hipSuccess;
  const int K = k0_host[n_groups];
  SharedGemmArgs a{act, w, nullptr, M, N, K, nullptr, out, static_cast<int64_t>(M) * N, nullptr, nullptr};
  if (static_cast<int64_t>((M + 255) / 256) * ((N + 255) / 256) * n_groups >= 256)
    return launch_kgrouped_cfg<SharedCfg<1, 2, 4, 4, 2, 1, 4>>(a, k0_host, n_groups, stream);   // 256 x 256
  return launch_kgrouped_cfg<SharedCfg<1, 2, 2, 2, 2, 2>>(a, k0_host, n_groups, stream);        // 128 x 128
}

}  // namespace mote
