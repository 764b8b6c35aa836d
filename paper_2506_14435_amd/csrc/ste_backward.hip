// Straight-through estimator of Section 3.2 for the grouped ternary linear layer of Section 3.1,
// Y_e = Q_a(X_e) Q_w(W_e)^T: the quantisers are skipped on the way back, so with the rows of dY
// grouped by expert
//
//   dX[r, c]   = alpha_e * sum_n dY[r, n] * t_e[n, c]
//   dW_e[n, c] = sum_{r in e} bf16(dY[r, n] * beta_r / 127) * q[r, c]
//
// Both are dense bf16 contractions with fp32 accumulation (ternary values and int8 codes are
// exact in bf16) and run on the bf16 MFMA GEMM of the shared expert, which contracts two
// row-major operands along their rows: dX of all experts as one launch over groups of rows, each
// with its own weight matrix; dW of all experts as one launch whose K ranges are the experts.  The
// kernels here bring the operands into that form, each in one launch over all experts:
//
//   expand_ternary_t_kernel : packed 2-bit codes of W_e [N, K] -> bf16 matrix [K, N] of t_e^T
//   transpose_groups_kernel : dY [R, N] bf16, scaled by beta_r / 127 and rounded once -> [N, sum_pad],
//                             q [R, K] int8 -> bf16 [K, sum_pad]; expert e in the columns pad0[e] ..,
//                             its rows rounded up to 64 with zeros
//   fill_alpha_kernel       : alpha_e broadcast over the K output channels of dX (the GEMM
//                             epilogue multiplies per output channel)
#include <algorithm>

#include "common.h"
#include "launch.h"

namespace mote {

constexpr int kSteThreads = 256;

// One workgroup expands four packed tiles (32 output rows x 128 input channels each, consecutive
// row tiles nt = 4 b .. 4 b + 3 of one K tile) into a 128 x 128 block of the transposed matrix:
// out[(128 kt + c) * N + 128 b + n] = t[128 b + n][128 kt + c].
__device__ __forceinline__ void expand_ternary_t_body(const uint32_t* __restrict__ packed, int N, int K,
                                                      uint16_t* __restrict__ out) {
  __shared__ uint16_t s_t[128][128 + 2];   // [c][n], two bf16 of padding per row
  const int tiles_k = K >> 7;
  const int kt = blockIdx.x % tiles_k, nb = blockIdx.x / tiles_k;
  const int tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int nt = nb * 4 + j;
    const uint32_t word = packed[(static_cast<int64_t>(nt) * tiles_k + kt) * 256 + tid];
    const int lane = tid >> 2, s = tid & 3;
    const int r = lane & 31, g = lane >> 5;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int code = (word >> (8 * (i & 3) + 2 * (i >> 2))) & 3;
      // t = code - 1 as bf16: -1 = 0xBF80, 0 = 0, +1 = 0x3F80
      s_t[32 * s + 16 * g + i][32 * j + r] = code == 1 ? 0 : (code == 0 ? 0xBF80 : 0x3F80);
    }
  }
  __syncthreads();
  // row c of the block: 128 bf16 = 256 bytes, written by 16 threads of 16 bytes
  for (int i = tid; i < 128 * 16; i += kSteThreads) {
    const int c = i >> 4, part = i & 15;
    u4 v;
    const uint16_t* src = &s_t[c][part * 8];
    v.x = src[0] | (static_cast<uint32_t>(src[1]) << 16);
    v.y = src[2] | (static_cast<uint32_t>(src[3]) << 16);
    v.z = src[4] | (static_cast<uint32_t>(src[5]) << 16);
    v.w = src[6] | (static_cast<uint32_t>(src[7]) << 16);
    *reinterpret_cast<u4*>(out + (static_cast<int64_t>(kt) * 128 + c) * N + nb * 128 + part * 8) = v;
  }
}

// Expert e0 + blockIdx.y of `packed` ([experts][N, K] packed) into matrix blockIdx.y of `out`; experts
// without rows (row0[e] == row0[e + 1]) are skipped, their matrices are never read.
struct SteGroups {
  int n;
  int row0[65];
  int col0[65];   // first column of the expert's block in the transposed operands (rows padded to 64 per expert)
};
__global__ __launch_bounds__(kSteThreads) void expand_ternary_t_kernel(const uint32_t* __restrict__ packed, int N, int K,
                                                                       SteGroups grp, int e0, uint16_t* __restrict__ out) {
  const int e = e0 + blockIdx.y;
  if (grp.row0[e] == grp.row0[e + 1]) return;
  expand_ternary_t_body(packed + static_cast<int64_t>(e) * (static_cast<int64_t>(N) * K / 16), N, K,
                        out + static_cast<int64_t>(blockIdx.y) * K * N);
}

// in [rows, C] (bf16 bit patterns scaled by beta[r] / 127, or int8 codes) -> out [C, ld] bf16, columns
// 0 .. rows_pad - 1 of it (the caller offsets `out` to the expert's first column), 64 x 64 tiles
// through LDS.  Rows from `rows` up to rows_pad are written as zeros.
template <bool INT8>
__device__ __forceinline__ void transpose_rows_body(const void* __restrict__ in, const float* __restrict__ beta, int rows,
                                                    int C, int64_t ld, uint16_t* __restrict__ out) {
  __shared__ uint16_t s_t[64][64 + 2];   // [c][r]
  const int c_tiles = C >> 6;
  const int ct = blockIdx.x % c_tiles, rt = blockIdx.x / c_tiles;
  const int tid = threadIdx.x;
  // load: thread t reads 16 consecutive channels of row rt * 64 + t / 4
  {
    const int r = rt * 64 + (tid >> 2), c0 = ct * 64 + (tid & 3) * 16;
    uint16_t v[16];
    if (r < rows) {
      if constexpr (INT8) {
        const u4 raw = *reinterpret_cast<const u4*>(static_cast<const int8_t*>(in) + static_cast<int64_t>(r) * C + c0);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int q = static_cast<int8_t>((w[i >> 2] >> (8 * (i & 3))) & 0xFF);
          v[i] = f32_to_bf16(static_cast<float>(q));   // |q| <= 128: exact
        }
      } else {
        const float s = beta[r] / 127.0f;   // the scale of Q_a, as the forward pass forms it
        const uint16_t* src = static_cast<const uint16_t*>(in) + static_cast<int64_t>(r) * C + c0;
        const u4 a = *reinterpret_cast<const u4*>(src), b = *reinterpret_cast<const u4*>(src + 8);
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          v[2 * i] = f32_to_bf16(bf16_lo(w[i]) * s);
          v[2 * i + 1] = f32_to_bf16(bf16_hi(w[i]) * s);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = 0;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) s_t[(tid & 3) * 16 + i][tid >> 2] = v[i];
  }
  __syncthreads();
  // store: thread t writes 16 consecutive rows of channel ct * 64 + t / 4
  {
    const int c = tid >> 2, r0 = (tid & 3) * 16;
    const uint16_t* src = &s_t[c][r0];
    u4 a, b;
    a.x = src[0] | (static_cast<uint32_t>(src[1]) << 16);
    a.y = src[2] | (static_cast<uint32_t>(src[3]) << 16);
    a.z = src[4] | (static_cast<uint32_t>(src[5]) << 16);
    a.w = src[6] | (static_cast<uint32_t>(src[7]) << 16);
    b.x = src[8] | (static_cast<uint32_t>(src[9]) << 16);
    b.y = src[10] | (static_cast<uint32_t>(src[11]) << 16);
    b.z = src[12] | (static_cast<uint32_t>(src[13]) << 16);
    b.w = src[14] | (static_cast<uint32_t>(src[15]) << 16);
    uint16_t* dst = out + static_cast<int64_t>(ct * 64 + c) * ld + rt * 64 + r0;
    *reinterpret_cast<u4*>(dst) = a;
    *reinterpret_cast<u4*>(dst + 8) = b;
  }
}

// Every expert in one launch (blockIdx.y = expert): expert e owns the rows row0[e] .. row0[e+1]-1
// of `in` and the columns col0[e] .. col0[e+1]-1 of `out` ([C, ld]; the block is padded with zeros to a
// multiple of 64 columns).  The grid covers the longest block; workgroups past an expert's block leave.
template <bool INT8>
__global__ __launch_bounds__(kSteThreads) void transpose_groups_kernel(const void* __restrict__ in, const float* __restrict__ beta,
                                                                       SteGroups grp, int C, int64_t ld, uint16_t* __restrict__ out) {
  const int e = blockIdx.y, r0 = grp.row0[e], c0 = grp.col0[e];
  if (static_cast<int>(blockIdx.x / (C >> 6)) * 64 >= grp.col0[e + 1] - c0) return;
  const void* const in_e = INT8 ? static_cast<const void*>(static_cast<const int8_t*>(in) + static_cast<int64_t>(r0) * C)
                                : static_cast<const void*>(static_cast<const uint16_t*>(in) + static_cast<int64_t>(r0) * C);
  transpose_rows_body<INT8>(in_e, INT8 ? nullptr : beta + r0, grp.row0[e + 1] - r0, C, ld, out + c0);
}

__global__ __launch_bounds__(kSteThreads) void fill_alpha_kernel(const float* __restrict__ alpha, int alpha_stride, int E,
                                                                 int K, float* __restrict__ out) {
  const int i = blockIdx.x * kSteThreads + threadIdx.x;
  if (i < E * K) out[i] = alpha[(i / K) * alpha_stride];
}

__global__ __launch_bounds__(kSteThreads) void fill_zero_kernel(float* __restrict__ out, int64_t n4) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kSteThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kSteThreads + threadIdx.x; i < n4; i += stride)
    reinterpret_cast<float4*>(out)[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}

// out[i] = scale * (plane 0 + plane 1 + ...)[i], planes added in order; alpha == nullptr: scale 1
__global__ __launch_bounds__(kSteThreads) void sum_planes_kernel(const float* __restrict__ planes, int n_planes, int64_t n4,
                                                                 const float* __restrict__ alpha, float* __restrict__ out) {
  const float scale = alpha != nullptr ? alpha[0] : 1.0f;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kSteThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kSteThreads + threadIdx.x; i < n4; i += stride) {
    float4 acc = reinterpret_cast<const float4*>(planes)[i];
    for (int p = 1; p < n_planes; ++p) {
      const float4 v = reinterpret_cast<const float4*>(planes)[p * n4 + i];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    reinterpret_cast<float4*>(out)[i] = make_float4(acc.x * scale, acc.y * scale, acc.z * scale, acc.w * scale);
  }
}

static inline size_t ste_align(size_t v) { return (v + 255) / 256 * 256; }

// K planes of the dX contraction at most; dX runs as one grouped GEMM over as many experts as have
// their expanded weights below 4 GiB together (the kernel addresses them with 32-bit byte offsets;
// the limit is a tuning knob so that tests reach the loop over batches with small matrices).
constexpr int kSteMaxPlanes = 8;
static int ste_dx_batch(int N, int K, int E) {
  const int64_t per = static_cast<int64_t>(N) * K * 2;
  const int64_t lim_mib = std::min(std::max(knob(kKnobSteBatchMiB), 1), 4095);
  const int64_t g = ((lim_mib << 20) + ((int64_t{1} << 20) - 1)) / per;
  return static_cast<int>(std::max<int64_t>(1, std::min<int64_t>(g, E)));
}

// Workspace: the expanded transposed weights of one batch of experts [experts][K, N], the transposed
// scaled gradient rows and codes of every expert (sum of rows_pad_e <= R + 63 E columns, a sixteenth
// more when near-equal blocks are padded to the longest), alpha
// broadcast [E, K], partial planes of dX.
static size_t ste_pad_rows(int R, int E) { return (static_cast<size_t>(R) + 64 * static_cast<size_t>(E)) * 17 / 16 + 64; }
size_t ste_backward_workspace_bytes(int R, int N, int K, int E) {
  const size_t rp = ste_pad_rows(R, E);
  const size_t plane_bytes = static_cast<size_t>(kSteMaxPlanes) * R * K * 4;
  return ste_align(static_cast<size_t>(ste_dx_batch(N, K, E)) * K * N * 2) + ste_align(rp * N * 2) + ste_align(rp * K * 2) +
         ste_align(static_cast<size_t>(E) * K * 4) + ste_align(plane_bytes);
}

hipError_t launch_ste_backward(const uint16_t* dy, const int32_t* offsets_host, const uint32_t* packed, const float* alpha,
                               int alpha_stride, const int8_t* q, const float* beta, int R, int N, int K, int E,
                               float* dx, float* dw, void* workspace, hipStream_t stream) {
  char* ws = static_cast<char*>(workspace);
  const size_t rp_total = ste_pad_rows(R, E);
  const int batch = ste_dx_batch(N, K, E);
  uint16_t* wt = reinterpret_cast<uint16_t*>(ws);
  ws += ste_align(static_cast<size_t>(batch) * K * N * 2);
  uint16_t* dyt = reinterpret_cast<uint16_t*>(ws);
  ws += ste_align(rp_total * N * 2);
  uint16_t* qt = reinterpret_cast<uint16_t*>(ws);
  ws += ste_align(rp_total * K * 2);
  float* alpha_vec = reinterpret_cast<float*>(ws);
  ws += ste_align(static_cast<size_t>(E) * K * 4);
  float* dx_planes = reinterpret_cast<float*>(ws);

  SteGroups grp;
  grp.n = E;
  int32_t pad0[65];   // first padded row of every expert = K ranges of the dW contraction
  int64_t sum_pad = 0, tight = 0;
  int longest = 0;
  for (int e = 0; e < E; ++e) {
    const int rows_pad = (offsets_host[e + 1] - offsets_host[e] + 63) / 64 * 64;
    tight += rows_pad;
    longest = std::max(longest, rows_pad);
  }
  // near-equal groups: every block as long as the longest (at most 1/16 more contraction steps); tiles of
  // equal length keep the workgroups of the dW GEMM in step (3B width, 16 groups of about 1024 rows:
  // 966 -> 921 us for the GEMM)
  const bool uniform = static_cast<int64_t>(E) * longest * 16 <= tight * 17;
  for (int e = 0; e <= 64; ++e) {
    grp.row0[e] = offsets_host[std::min(e, E)];
    grp.col0[e] = pad0[e] = static_cast<int32_t>(sum_pad);
    if (e < E) sum_pad += uniform ? longest : (offsets_host[e + 1] - offsets_host[e] + 63) / 64 * 64;
  }

  fill_alpha_kernel<<<(E * K + kSteThreads - 1) / kSteThreads, kSteThreads, 0, stream>>>(alpha, alpha_stride, E, K, alpha_vec);
  // dX: t^T of a batch of experts expanded to bf16, then one grouped GEMM over their rows, scaled by alpha
  for (int e0 = 0; e0 < E; e0 += batch) {
    const int nb = std::min(batch, E - e0);
    const int row0 = offsets_host[e0], rows = offsets_host[e0 + nb] - row0;
    if (rows == 0) continue;
    expand_ternary_t_kernel<<<dim3((N / 128) * (K / 128), nb), kSteThreads, 0, stream>>>(packed, N, K, grp, e0, wt);
    const int planes = grouped_gemm_planes(offsets_host + e0, nb, K, N, kSteMaxPlanes);
    const uint16_t* dy_b = dy + static_cast<int64_t>(row0) * N;
    float* dx_b = dx + static_cast<int64_t>(row0) * K;
    const float* alpha_b = alpha_vec + static_cast<int64_t>(e0) * K;
    hipError_t err = launch_gemm_grouped_f32(dy_b, wt, offsets_host + e0, nb, K, N, planes == 1 ? dx_b : dx_planes, alpha_b,
                                             planes, stream);
    if (err != hipSuccess) return err;
    if (planes > 1) {   // the contraction over N was cut into planes, added in order here
      const int64_t n4 = static_cast<int64_t>(rows) * K / 4;
      sum_planes_kernel<<<static_cast<unsigned>(std::min<int64_t>((n4 + kSteThreads - 1) / kSteThreads, 2048)), kSteThreads,
                          0, stream>>>(dx_planes, planes, n4, nullptr, dx_b);
    }
  }
  // dW: the scaled gradient rows and the codes of every expert transposed into [N, sum_pad] and [K, sum_pad]
  // (expert e in the columns pad0[e] .., padded with zeros to a multiple of 64), then ONE GEMM whose K
  // ranges are the experts: plane e = dW_e, zeros for an expert without rows.
  if (sum_pad == 0) {
    fill_zero_kernel<<<1024, kSteThreads, 0, stream>>>(dw, static_cast<int64_t>(E) * N * K / 4);
    return hipGetLastError();
  }
  const unsigned tiles_r = static_cast<unsigned>(longest / 64);
  transpose_groups_kernel<false><<<dim3(tiles_r * (N / 64), E), kSteThreads, 0, stream>>>(dy, beta, grp, N, sum_pad, dyt);
  transpose_groups_kernel<true><<<dim3(tiles_r * (K / 64), E), kSteThreads, 0, stream>>>(q, nullptr, grp, K, sum_pad, qt);
  hipError_t err = launch_gemm_tn_f32_kgroups(dyt, qt, N, K, pad0, E, dw, stream);
  if (err != hipSuccess) return err;
  return hipGetLastError();
}

}  // namespace mote
