// Shared expert FFN(x) of Eq.2: the dense checkpoint's full-precision SwiGLU FFN, active
// for every token.  bf16 operands on v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
//   gate-up mode : g = x W_gate^T, u = x W_up^T, h_s = bf16(u * SiLU(g))     [T, F]
//   down mode    : y_s = h_s W_down^T (fp32)                                 [T, d]
//
// Both operands are K-contiguous ([rows, K] row-major), so a tile row is 64 bf16 = 128
// bytes and the LDS geometry (8 XOR-swizzled 16-byte chunks per row) is the same for the
// activation and the weight tiles.  MFMA operand mapping: first operand = weights (lane l:
// output channel l%32, 8 consecutive K elements of half l/32), second = activations (lane
// l: token row l%32); result register v of lane l is output channel 8*(v/4) + 4*(l/32) +
// v%4 of token row l%32.
#include <stdlib.h>

#include "common.h"
#include "launch.h"

namespace mote {

template <int MODE_, int BM_W_, int BN_W_, int WAVES_M_, int WAVES_N_, int MIN_BLOCKS_ = 1>
struct SharedCfg {
  static constexpr int MIN_BLOCKS = MIN_BLOCKS_;
  static constexpr int MODE = MODE_;
  static constexpr int NMAT = MODE_ == 0 ? 2 : 1;
  static constexpr int BM_W = BM_W_, BN_W = BN_W_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int BM = 32 * BM_W_ * WAVES_M_;
  static constexpr int BN = 32 * BN_W_ * WAVES_N_;
  static constexpr int THREADS = 64 * WAVES_M_ * WAVES_N_;
  static constexpr int ROWS_PER_PASS = THREADS / 8;
  static constexpr int A_PASSES = BM / ROWS_PER_PASS;
  static constexpr int B_PASSES = BN / ROWS_PER_PASS;
  static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "loaders cover the tiles in whole passes");
  static constexpr int A_BYTES = BM * 128;
  static constexpr int B_BYTES = BN * 128;
  static constexpr int STAGE_BYTES = A_BYTES + NMAT * B_BYTES;
};

// 128-byte rows of eight 16-byte chunks, chunk XOR-swizzled with row bits 1..3: 16 lanes
// reading one chunk of 16 consecutive rows cover all 64 LDS banks exactly once.
__device__ __forceinline__ int lds_tile_offset(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

struct SharedGemmArgs {
  const uint16_t* act;   // [M, K] bf16
  const uint16_t* w0;    // [N, K] bf16 (gate / down)
  const uint16_t* w1;    // [N, K] bf16 (up)
  int M, N, K;
  uint16_t* h_out;       // gate-up: bf16 [M, N]
  float* y_out;          // down: fp32 [planes][M, N]
  int64_t plane_stride;  // elements between partial planes
};

template <typename Cfg>
__global__ __launch_bounds__(Cfg::THREADS, Cfg::MIN_BLOCKS) void shared_gemm_kernel(SharedGemmArgs a, int n_ntiles, int kplanes, int ktp) {
  constexpr int NMAT = Cfg::NMAT, BM_W = Cfg::BM_W, BN_W = Cfg::BN_W;
  constexpr int BM = Cfg::BM, BN = Cfg::BN;
  extern __shared__ __attribute__((aligned(16))) unsigned char s_mem[];

  // Workgroups go to the 8 XCDs round-robin by linear id: XCD x owns the channel tiles
  // x, x+8, ... (the row tiles x, x+8, ... when there are fewer than 16 channel tiles) and
  // walks the other index fastest, so its L2 keeps one slice of the weights resident.
  // With kplanes > 1 (down projection of small problems) the contraction is cut into planes of
  // ktp K steps; each plane writes its own partial output, added later in plane order.
  n_ntiles *= kplanes;
  const int M = a.M, N = a.N, K = a.K;
  const int n_mtiles = (M + BM - 1) / BM;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const bool split_n = n_ntiles >= 16;
  const int xcd_ntiles = split_n ? (n_ntiles - xcd + 7) >> 3 : n_ntiles;
  const int xcd_mtiles = split_n ? n_mtiles : (n_mtiles - xcd + 7) >> 3;
  if (slot >= xcd_ntiles * xcd_mtiles) return;
  const int mi = slot / xcd_ntiles, ni = slot - mi * xcd_ntiles;
  const int mt = split_n ? mi : xcd + 8 * mi;
  const int ntk = split_n ? xcd + 8 * ni : ni;
  const int nt = ntk / kplanes, kc = ntk - nt * kplanes;
  const int kt0 = kc * ktp;
  const int KT = min(ktp, (K >> 6) - kt0);   // K steps of this plane
  const int m0 = mt * BM, n0 = nt * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int r32 = lane & 31, g = lane >> 5;
  const int chunk = tid & 7;

  const uint16_t* a_src[Cfg::A_PASSES];
  const uint16_t* b_src[NMAT][Cfg::B_PASSES];
  int a_dst[Cfg::A_PASSES], b_dst[Cfg::B_PASSES];
#pragma unroll
  for (int p = 0; p < Cfg::A_PASSES; ++p) {
    const int r = p * Cfg::ROWS_PER_PASS + (tid >> 3);
    a_src[p] = a.act + static_cast<int64_t>(min(m0 + r, M - 1)) * K + chunk * 8 + kt0 * 64;
    a_dst[p] = lds_tile_offset(r, chunk);
  }
#pragma unroll
  for (int p = 0; p < Cfg::B_PASSES; ++p) {
    const int r = p * Cfg::ROWS_PER_PASS + (tid >> 3);
    const int64_t off = static_cast<int64_t>(min(n0 + r, N - 1)) * K + chunk * 8 + kt0 * 64;
    b_src[0][p] = a.w0 + off;
    if constexpr (NMAT == 2) b_src[1][p] = a.w1 + off;
    b_dst[p] = lds_tile_offset(r, chunk);
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

  u4 a_reg[Cfg::A_PASSES], b_reg[NMAT][Cfg::B_PASSES];

#define MOTE_GLOAD(kt_)                                                                              \
  do {                                                                                             \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                                      \
      a_reg[p] = *reinterpret_cast<const u4*>(a_src[p] + static_cast<int64_t>(kt_) * 64);        \
    _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                               \
      _Pragma("unroll") for (int p = 0; p < Cfg::B_PASSES; ++p)                                    \
        b_reg[m][p] = *reinterpret_cast<const u4*>(b_src[m][p] + static_cast<int64_t>(kt_) * 64); \
  } while (0)
#define MOTE_LSTORE(stage_idx_)                                                                    \
  do {                                                                                             \
    unsigned char* st_ = s_mem + (stage_idx_) * Cfg::STAGE_BYTES;                                  \
    _Pragma("unroll") for (int p = 0; p < Cfg::A_PASSES; ++p)                                      \
      *reinterpret_cast<u4*>(st_ + a_dst[p]) = a_reg[p];                                        \
    _Pragma("unroll") for (int m = 0; m < NMAT; ++m)                                               \
      _Pragma("unroll") for (int p = 0; p < Cfg::B_PASSES; ++p)                                    \
        *reinterpret_cast<u4*>(st_ + Cfg::A_BYTES + m * Cfg::B_BYTES + b_dst[p]) = b_reg[m][p]; \
  } while (0)

  MOTE_GLOAD(0);
  MOTE_LSTORE(0);
  __syncthreads();

  const int a_row_base = wm * BM_W * 32 + r32;
  const int b_row_base = wn * BN_W * 32 + r32;
  for (int kt = 0; kt < KT; ++kt) {
    const bool has_next = kt + 1 < KT;
    if (has_next) MOTE_GLOAD(kt + 1);
    __builtin_amdgcn_sched_barrier(0);  // keep the prefetch loads ahead of the contraction
    const unsigned char* st = s_mem + (kt & 1) * Cfg::STAGE_BYTES;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 af[BM_W];
#pragma unroll
      for (int i = 0; i < BM_W; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(st + lds_tile_offset(a_row_base + i * 32, 2 * s + g));
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < BN_W; ++f) {
          const bf16x8 bf = *reinterpret_cast<const bf16x8*>(st + Cfg::A_BYTES + m * Cfg::B_BYTES +
                                                             lds_tile_offset(b_row_base + f * 32, 2 * s + g));
#pragma unroll
          for (int i = 0; i < BM_W; ++i)
            acc[m][i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, af[i], acc[m][i][f], 0, 0, 0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (has_next) MOTE_LSTORE((kt + 1) & 1);
    __syncthreads();
  }

#undef MOTE_GLOAD
#undef MOTE_LSTORE

  // Lane l owns token row r32 of every row fragment and runs of four consecutive output
  // channels (first MFMA operand = weights).
#pragma unroll
  for (int i = 0; i < BM_W; ++i) {
    const int row = m0 + wm * BM_W * 32 + i * 32 + r32;
    if (row >= M) continue;
#pragma unroll
    for (int f = 0; f < BN_W; ++f) {
      const int nf = n0 + wn * BN_W * 32 + f * 32;
      if (nf >= N) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int64_t o = static_cast<int64_t>(row) * N + nf + 8 * q + 4 * g;
        if constexpr (Cfg::MODE == 0) {
          float hv[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) hv[j] = acc[1][i][f][4 * q + j] * silu_fast(acc[0][i][f][4 * q + j]);
          uint2 packed;
          packed.x = cvt_pk_bf16(hv[0], hv[1]);
          packed.y = cvt_pk_bf16(hv[2], hv[3]);
          *reinterpret_cast<uint2*>(a.h_out + o) = packed;
        } else {
          *reinterpret_cast<float4*>(a.y_out + static_cast<int64_t>(kc) * a.plane_stride + o) = make_float4(acc[0][i][f][4 * q + 0], acc[0][i][f][4 * q + 1],
                                                                acc[0][i][f][4 * q + 2], acc[0][i][f][4 * q + 3]);
        }
      }
    }
  }
}

// Largest per-XCD tile count of the XCD-aware mapping (XCD 0 owns the most tiles).
static int split_tiles(int n_ntiles, int n_mtiles) {
  return n_ntiles >= 16 ? ((n_ntiles + 7) / 8) * n_mtiles : n_ntiles * ((n_mtiles + 7) / 8);
}

static int shared_variant() {
  static int v = -1;
  if (v < 0) {
    const char* e = getenv("MOTE_SHARED_VARIANT");
    v = e ? atoi(e) : 0;
  }
  return v;
}

template <typename Cfg>
static hipError_t launch_shared_cfg(const SharedGemmArgs& a, int kplanes, hipStream_t stream) {
  const int n_ntiles = (a.N + Cfg::BN - 1) / Cfg::BN;
  const int KT = a.K >> 6;
  const int ktp = (KT + kplanes - 1) / kplanes;
  const int n_mtiles = (a.M + Cfg::BM - 1) / Cfg::BM;
  const size_t lds = 2 * Cfg::STAGE_BYTES;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(shared_gemm_kernel<Cfg>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int per_xcd = split_tiles(n_ntiles * kplanes, n_mtiles);
  shared_gemm_kernel<Cfg><<<static_cast<unsigned>(per_xcd * 8), Cfg::THREADS, lds, stream>>>(a, n_ntiles, kplanes, ktp);
  return hipGetLastError();
}

hipError_t launch_shared_gate_up(const uint16_t* x, const uint16_t* w_gate, const uint16_t* w_up, int T, int d,
                                 int F, uint16_t* h_s, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  SharedGemmArgs a{x, w_gate, w_up, T, F, d, h_s, nullptr, 0};
  int v = shared_variant();
  if (v == 0) {   // few 256-row tiles: the 128 x (64+64) tile at two workgroups per CU fills the chip better
    const int64_t big_tiles = static_cast<int64_t>((T + 255) / 256) * (F / 128);
    if (big_tiles < 2 * 256) v = 1;
  }
  switch (v) {
    case 1: return launch_shared_cfg<SharedCfg<0, 2, 1, 2, 2, 2>>(a, 1, stream);   // 128 x (64+64), 2 workgroups / CU
    case 2: return launch_shared_cfg<SharedCfg<0, 2, 2, 2, 2, 1>>(a, 1, stream);   // 128 x (128+128), 1 workgroup / CU
    default: return launch_shared_cfg<SharedCfg<0, 2, 2, 4, 2, 1>>(a, 1, stream);  // 256 x (128+128), 8 wavefronts
  }
}

// K planes of the large-batch down projection: enough (row tile, channel tile, plane) triples
// to fill two workgroups per CU, planes of at least 8 K steps.  Pure function of the shape:
// the workspace layout depends on it.
int shared_down_planes(int T, int d, int F) {
  const int64_t tiles = static_cast<int64_t>((T + 127) / 128) * ((d + 127) / 128);
  const int KT = F >> 6;
  int planes = static_cast<int>(512 / (tiles > 0 ? tiles : 1));
  if (planes > 8) planes = 8;
  if (planes > KT / 8) planes = KT / 8;
  if (planes < 1) planes = 1;
  const int ktp = (KT + planes - 1) / planes;
  return (KT + ktp - 1) / ktp;
}

hipError_t launch_shared_down(const uint16_t* h_s, const uint16_t* w_down, int T, int d, int F, float* y_s,
                              hipStream_t stream) {
  if (T == 0) return hipSuccess;
  SharedGemmArgs a{h_s, w_down, nullptr, T, d, F, nullptr, y_s, static_cast<int64_t>(T) * d};
  const int planes = shared_down_planes(T, d, F);
  switch (shared_variant()) {
    case 1: return launch_shared_cfg<SharedCfg<1, 2, 4, 2, 2, 1>>(a, planes, stream);   // 128 x 256
    case 2: return launch_shared_cfg<SharedCfg<1, 4, 2, 2, 2, 1>>(a, planes, stream);   // 256 x 128
    default: return launch_shared_cfg<SharedCfg<1, 2, 2, 2, 2, 2>>(a, planes, stream);  // 128 x 128, 2 workgroups / CU
  }
}

}  // namespace mote
