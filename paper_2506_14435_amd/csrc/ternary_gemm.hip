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
// into the four B-operand registers of one v_mfma_i32_32x32x32_i8.  The codes are t+1, so
// the accumulator holds sum (t+1) q; the row sum of q is subtracted in the epilogue.
//
// MFMA operand mapping (32x32x32 i8): A = activations, lane l supplies row l%32, 16
// consecutive channels of half l/32; B = weights, lane l supplies output channel l%32,
// the same 16 channels.  Result register v of lane l is row 8*(v/4) + 4*(l/32) + v%4,
// output channel l%32.
#include "common.h"
#include "launch.h"

namespace mote {

template <int MODE_, int BM_W_, int BN_W_, int WAVES_M_, int WAVES_N_>
struct RoutedCfg {
  static constexpr int MODE = MODE_;  // 0 gate-up (two matrices, SwiGLU epilogue), 1 down
  static constexpr int NMAT = MODE_ == 0 ? 2 : 1;
  static constexpr int BM_W = BM_W_, BN_W = BN_W_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int BM = 32 * BM_W_ * WAVES_M_;
  static constexpr int BN = 32 * BN_W_ * WAVES_N_;
  static constexpr int THREADS = 64 * WAVES_M_ * WAVES_N_;
  static constexpr int ROWS_PER_PASS = THREADS / 8;
  static constexpr int A_PASSES = BM / ROWS_PER_PASS;
  static constexpr int STAGE_BYTES = BM * 128;
  static_assert(BM % ROWS_PER_PASS == 0, "activation loader covers the tile in whole passes");
};

__device__ __forceinline__ v4i unpack_codes(uint32_t w) {
  v4i b;
  b.x = static_cast<int>(w & 0x03030303u);
  b.y = static_cast<int>((w >> 2) & 0x03030303u);
  b.z = static_cast<int>((w >> 4) & 0x03030303u);
  b.w = static_cast<int>((w >> 6) & 0x03030303u);
  return b;
}

__device__ __forceinline__ int lds_a_offset(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }

template <typename Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void routed_gemm_kernel(RoutedGemmArgs a, int n_ntiles) {
  constexpr int NMAT = Cfg::NMAT, BM_W = Cfg::BM_W, BN_W = Cfg::BN_W;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, THREADS = Cfg::THREADS;
  __shared__ __attribute__((aligned(16))) unsigned char s_a[2 * Cfg::STAGE_BYTES];
  __shared__ float s_scale[BM];
  __shared__ int s_rs[BM];

  const int nt = blockIdx.x % n_ntiles;
  const int mt = blockIdx.x / n_ntiles;
  if (mt >= a.plan.n_tiles[0]) return;
  const int expert = a.plan.tile_expert[mt];
  const int row0 = a.plan.tile_row0[mt];
  const int rows = a.plan.tile_rows[mt];
  const int K = a.K, N = a.N;
  const int KT = K >> 7;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int r32 = lane & 31, g = lane >> 5;

  // ---- per-row metadata (scale = beta/127, row sum) ----
  for (int r = tid; r < BM; r += THREADS) {
    const int slot = row0 + min(r, rows - 1);
    const int src = a.gather ? a.gather[slot] : slot;
    s_scale[r] = a.beta[src] / 127.0f;
    s_rs[r] = a.rowsum[src];
  }

  // ---- activation loader: thread -> (row, 16-byte chunk) per pass ----
  const int8_t* a_src[Cfg::A_PASSES];
  int a_dst[Cfg::A_PASSES];
  {
    const int chunk = tid & 7;
#pragma unroll
    for (int p = 0; p < Cfg::A_PASSES; ++p) {
      const int r = p * Cfg::ROWS_PER_PASS + (tid >> 3);
      const int slot = row0 + min(r, rows - 1);
      const int src = a.gather ? a.gather[slot] : slot;
      a_src[p] = a.q + static_cast<int64_t>(src) * K + chunk * 16;
      a_dst[p] = lds_a_offset(r, chunk);
    }
  }

  // ---- weight stream: one 16-byte load per lane per (matrix, fragment) per K step ----
  const int n_wave0 = nt * BN + wn * BN_W * 32;  // first output channel of this wavefront
  const u4* w_ptr[NMAT][BN_W];
  bool f_valid[BN_W];
  {
    const int64_t expert_words = static_cast<int64_t>(N) * K / 16;
#pragma unroll
    for (int f = 0; f < BN_W; ++f) {
      const int n_frag = n_wave0 + f * 32;
      f_valid[f] = n_frag < N;
      const int nt32 = (f_valid[f] ? n_frag : 0) >> 5;
      const int64_t off = static_cast<int64_t>(expert) * expert_words + static_cast<int64_t>(nt32) * KT * 256 + lane * 4;
      w_ptr[0][f] = reinterpret_cast<const u4*>(a.w_gate + off);
      if constexpr (NMAT == 2) w_ptr[1][f] = reinterpret_cast<const u4*>(a.w_up + off);
    }
  }

  v16i acc[NMAT][BM_W][BN_W];
#pragma unroll
  for (int m = 0; m < NMAT; ++m)
#pragma unroll
    for (int i = 0; i < BM_W; ++i)
#pragma unroll
      for (int f = 0; f < BN_W; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[m][i][f][v] = 0;

  u4 w_cur[NMAT][BN_W], w_nxt[NMAT][BN_W];
  u4 a_reg[Cfg::A_PASSES];

  // prologue: K step 0
#pragma unroll
  for (int p = 0; p < Cfg::A_PASSES; ++p) a_reg[p] = *reinterpret_cast<const u4*>(a_src[p]);
#pragma unroll
  for (int m = 0; m < NMAT; ++m)
#pragma unroll
    for (int f = 0; f < BN_W; ++f) w_cur[m][f] = w_ptr[m][f][0];
#pragma unroll
  for (int p = 0; p < Cfg::A_PASSES; ++p) *reinterpret_cast<u4*>(s_a + a_dst[p]) = a_reg[p];
  __syncthreads();

  const int a_row_base = wm * BM_W * 32 + r32;
  for (int kt = 0; kt < KT; ++kt) {
    const bool has_next = kt + 1 < KT;
    if (has_next) {
#pragma unroll
      for (int p = 0; p < Cfg::A_PASSES; ++p)
        a_reg[p] = *reinterpret_cast<const u4*>(a_src[p] + static_cast<int64_t>(kt + 1) * 128);
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < BN_W; ++f) w_nxt[m][f] = w_ptr[m][f][static_cast<int64_t>(kt + 1) * 64];
    }
    const unsigned char* stage = s_a + (kt & 1) * Cfg::STAGE_BYTES;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      v4i af[BM_W];
#pragma unroll
      for (int i = 0; i < BM_W; ++i)
        af[i] = *reinterpret_cast<const v4i*>(stage + lds_a_offset(a_row_base + i * 32, 2 * s + g));
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
#pragma unroll
        for (int f = 0; f < BN_W; ++f) {
          const uint32_t word = s == 0 ? w_cur[m][f].x : s == 1 ? w_cur[m][f].y : s == 2 ? w_cur[m][f].z : w_cur[m][f].w;
          const v4i bf = unpack_codes(word);
#pragma unroll
          for (int i = 0; i < BM_W; ++i)
            acc[m][i][f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf, acc[m][i][f], 0, 0, 0);
        }
    }
    if (has_next) {
      unsigned char* nstage = s_a + ((kt + 1) & 1) * Cfg::STAGE_BYTES;
#pragma unroll
      for (int p = 0; p < Cfg::A_PASSES; ++p) *reinterpret_cast<u4*>(nstage + a_dst[p]) = a_reg[p];
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < NMAT; ++m)
#pragma unroll
      for (int f = 0; f < BN_W; ++f) w_cur[m][f] = w_nxt[m][f];
  }

  // ---- epilogue ----
  float al0 = a.alpha[expert * 3 + (Cfg::MODE == 0 ? 0 : 2)];
  float al1 = Cfg::MODE == 0 ? a.alpha[expert * 3 + 1] : 0.0f;
#pragma unroll
  for (int i = 0; i < BM_W; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = wm * BM_W * 32 + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
      if (rl >= rows) continue;
      const int rs = s_rs[rl];
      const int64_t out_row = static_cast<int64_t>(row0 + rl) * N;
#pragma unroll
      for (int f = 0; f < BN_W; ++f) {
        if (!f_valid[f]) continue;
        const int n = n_wave0 + f * 32 + r32;
        if constexpr (Cfg::MODE == 0) {
          const float sx = s_scale[rl];
          const int gi = acc[0][i][f][v] - rs, ui = acc[1][i][f][v] - rs;
          const float gv = static_cast<float>(gi) * (sx * al0);
          const float uv = static_cast<float>(ui) * (sx * al1);
          const float hv = uv * (gv / (1.0f + expf(-gv)));
          a.h[out_row + n] = f32_to_bf16(hv);
          if (a.tap_gate) a.tap_gate[out_row + n] = gi;
          if (a.tap_up) a.tap_up[out_row + n] = ui;
        } else {
          a.acc_out[out_row + n] = acc[0][i][f][v] - rs;
        }
      }
    }
  }
}

template <typename Cfg>
static hipError_t launch_cfg(const RoutedGemmArgs& a, hipStream_t stream) {
  const int n_ntiles = (a.N + Cfg::BN - 1) / Cfg::BN;
  const int64_t blocks = static_cast<int64_t>(a.max_tiles) * n_ntiles;
  routed_gemm_kernel<Cfg><<<static_cast<unsigned>(blocks), Cfg::THREADS, 0, stream>>>(a, n_ntiles);
  return hipGetLastError();
}

// Plan tile height: 32-row tiles when experts see few rows (decode), 128 otherwise.
int routed_tile_m(int T, int k, int E) {
  const int64_t avg = (static_cast<int64_t>(T) * k + E - 1) / E;
  return avg <= 48 ? 32 : 128;
}

hipError_t launch_routed_gate_up(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  if (a.tile_m == 32) return launch_cfg<RoutedCfg<0, 1, 1, 1, 4>>(a, stream);
  return launch_cfg<RoutedCfg<0, 2, 2, 2, 2>>(a, stream);
}

hipError_t launch_routed_down(const RoutedGemmArgs& a, hipStream_t stream) {
  if (a.max_tiles == 0) return hipSuccess;
  if (a.tile_m == 32) return launch_cfg<RoutedCfg<1, 1, 1, 1, 4>>(a, stream);
  return launch_cfg<RoutedCfg<1, 2, 2, 2, 2>>(a, stream);
}

}  // namespace mote
