// Pieces around the layer of Section 3.1:
//   * norm_rows_kernel       LN(.) of Eq.1-2 as RMSNorm (the Qwen2.5 base models) or layer normalisation,
//                            the prologue of the block x_l = x^a + MoE(LN(x^a)) + FFN(LN(x^a))
//   * balance_kernel         load-balancing statistic of Section 3.3, Eq.12
//   * rtn_pack_kernel        round-to-nearest INT8 / INT4 weight quantiser for the shared expert
//                            (Section 4.3, Table 3) and its packed storage
//   * rtn_dequant_kernel     packed codes -> integer-valued bf16 matrix (exact), the operand of the
//                            large-batch shared GEMM whose epilogue applies the row scales
#include "common.h"
#include "launch.h"

namespace mote {

// ------------------------------------------------------------------------------ norms
// One workgroup per token row.  Statistics and the normalised value are computed in fp64 (the
// row is re-read from L1/L2; nothing here is bandwidth critical) so that the single rounding to
// bf16 agrees with a double-precision evaluation except for ties closer than 1e-15.
constexpr int kNormThreads = 256;

__device__ __forceinline__ double block_sum(double v, double* s_part) {
  v = wave_sum(v);
  __syncthreads();   // s_part may still be read from a previous reduction
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int i = 0; i < kNormThreads / kWave; ++i) t += s_part[i];
  return t;
}

// kind 1: y = x / sqrt(mean x^2 + eps) * gamma;  kind 2: y = (x - mean) / sqrt(var + eps) * gamma + beta
__global__ __launch_bounds__(kNormThreads) void norm_rows_kernel(const uint16_t* __restrict__ x,
                                                                 const uint16_t* __restrict__ gamma,
                                                                 const uint16_t* __restrict__ beta, int kind, double eps,
                                                                 int d, uint16_t* __restrict__ y) {
  __shared__ double s_part[kNormThreads / kWave];
  const uint16_t* row = x + static_cast<int64_t>(blockIdx.x) * d;
  uint16_t* out = y + static_cast<int64_t>(blockIdx.x) * d;
  const int chunks = d >> 3;
  double mean = 0.0;
  if (kind == 2) {
    double s = 0.0;
    for (int ch = threadIdx.x; ch < chunks; ch += kNormThreads) {
      const uint4 p = *reinterpret_cast<const uint4*>(row + (ch << 3));
      s += static_cast<double>(bf16_lo(p.x)) + static_cast<double>(bf16_hi(p.x)) + static_cast<double>(bf16_lo(p.y)) +
           static_cast<double>(bf16_hi(p.y)) + static_cast<double>(bf16_lo(p.z)) + static_cast<double>(bf16_hi(p.z)) +
           static_cast<double>(bf16_lo(p.w)) + static_cast<double>(bf16_hi(p.w));
    }
    mean = block_sum(s, s_part) / d;
  }
  double sq = 0.0;
  for (int ch = threadIdx.x; ch < chunks; ch += kNormThreads) {
    const uint4 p = *reinterpret_cast<const uint4*>(row + (ch << 3));
    const float f[8] = {bf16_lo(p.x), bf16_hi(p.x), bf16_lo(p.y), bf16_hi(p.y), bf16_lo(p.z), bf16_hi(p.z), bf16_lo(p.w), bf16_hi(p.w)};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const double c = static_cast<double>(f[i]) - mean;
      sq = fma(c, c, sq);
    }
  }
  const double var = block_sum(sq, s_part) / d;
  const double r = sqrt(var + eps);
  for (int ch = threadIdx.x; ch < chunks; ch += kNormThreads) {
    const uint4 p = *reinterpret_cast<const uint4*>(row + (ch << 3));
    const uint4 gq = *reinterpret_cast<const uint4*>(gamma + (ch << 3));
    uint4 bq = make_uint4(0u, 0u, 0u, 0u);
    if (kind == 2) bq = *reinterpret_cast<const uint4*>(beta + (ch << 3));
    const float f[8] = {bf16_lo(p.x), bf16_hi(p.x), bf16_lo(p.y), bf16_hi(p.y), bf16_lo(p.z), bf16_hi(p.z), bf16_lo(p.w), bf16_hi(p.w)};
    const float gm[8] = {bf16_lo(gq.x), bf16_hi(gq.x), bf16_lo(gq.y), bf16_hi(gq.y), bf16_lo(gq.z), bf16_hi(gq.z), bf16_lo(gq.w), bf16_hi(gq.w)};
    const float bt[8] = {bf16_lo(bq.x), bf16_hi(bq.x), bf16_lo(bq.y), bf16_hi(bq.y), bf16_lo(bq.z), bf16_hi(bq.z), bf16_lo(bq.w), bf16_hi(bq.w)};
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // the same operations in the same order as the definition: ((x - mean) / r) * gamma + beta
      double v = (static_cast<double>(f[i]) - mean) / r * static_cast<double>(gm[i]);
      if (kind == 2) v += static_cast<double>(bt[i]);
      o[i] = static_cast<float>(v);
    }
    uint4 ob;
    ob.x = cvt_pk_bf16(o[0], o[1]); ob.y = cvt_pk_bf16(o[2], o[3]);
    ob.z = cvt_pk_bf16(o[4], o[5]); ob.w = cvt_pk_bf16(o[6], o[7]);
    *reinterpret_cast<uint4*>(out + (ch << 3)) = ob;
  }
}

hipError_t launch_norm_rows(const uint16_t* x, const uint16_t* gamma, const uint16_t* beta, int kind, double eps, int T,
                            int d, uint16_t* y, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  norm_rows_kernel<<<T, kNormThreads, 0, stream>>>(x, gamma, beta, kind, eps, d, y);
  return hipGetLastError();
}

// --------------------------------------------------------------- load balancing (Eq.12)
// One workgroup: wavefront w sums the gate probabilities of experts w, w+16, ... over all tokens
// in fp64 (fixed order: lane-strided partial sums, then the butterfly), then thread 0 forms
// L = E/|X| * sum_i t_i * sum_x P(x)_i with t_i the routed counts.
__global__ __launch_bounds__(1024) void balance_kernel(const float* __restrict__ gate_p, const int32_t* __restrict__ counts,
                                                       int T, int E, float* __restrict__ gate_p_sum,
                                                       float* __restrict__ loss) {
  __shared__ double s_sum[64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int e = wave; e < E; e += 16) {
    double acc = 0.0;
    for (int t = lane; t < T; t += 64) acc += static_cast<double>(gate_p[static_cast<int64_t>(t) * E + e]);
    acc = wave_sum(acc);
    if (lane == 0) s_sum[e] = acc;
  }
  __syncthreads();
  if (threadIdx.x < E) gate_p_sum[threadIdx.x] = static_cast<float>(s_sum[threadIdx.x]);
  if (threadIdx.x == 0) {
    double l = 0.0;
    for (int e = 0; e < E; ++e) l += static_cast<double>(counts[e]) * s_sum[e];
    loss[0] = static_cast<float>(static_cast<double>(E) / static_cast<double>(T) * l);
  }
}

hipError_t launch_balance(const float* gate_p, const int32_t* counts, int T, int E, float* gate_p_sum, float* loss,
                          hipStream_t stream) {
  balance_kernel<<<1, 1024, 0, stream>>>(gate_p, counts, T, E, gate_p_sum, loss);
  return hipGetLastError();
}

// ------------------------------------------------------------------ RTN (Section 4.3)
// Storage position p of a packed row -> input channel (see include/mote.h).  INT8: groups of 32,
// position 16g + 8a + i holds channel 16a + 8g + i; INT4: groups of 64, position 32g + 8s + i holds
// channel 16s + 8g + i.  Both make the 16 bytes a lane of the decode kernel reads from a row the
// operands of consecutive MFMAs for its K half g.
template <int BITS>
__device__ __forceinline__ int rtn_channel_of(int p) {
  if constexpr (BITS == 8) {
    const int grp = p >> 5, w = p & 31;
    return (grp << 5) + 16 * ((w >> 3) & 1) + 8 * (w >> 4) + (w & 7);
  } else {
    const int grp = p >> 6, w = p & 63;
    return (grp << 6) + 16 * ((w >> 3) & 3) + 8 * (w >> 5) + (w & 7);
  }
}

constexpr int kRtnThreads = 256;

// One workgroup per output row: absmax -> s = max(amax, 1e-5) / qmax (fp32 divide) ->
// q = clip(round_half_even(w / s), -qmax, qmax) (fp32 divide) -> two's-complement codes in
// storage order.  A thread writes 16 bytes (16 or 32 codes) per step.
template <int BITS>
__global__ __launch_bounds__(kRtnThreads) void rtn_pack_kernel(const uint16_t* __restrict__ w, int K,
                                                               unsigned char* __restrict__ packed,
                                                               float* __restrict__ scales) {
  __shared__ float s_max[kRtnThreads / kWave];
  constexpr float qmax = BITS == 8 ? 127.0f : 7.0f;
  constexpr int PER = BITS == 8 ? 16 : 32;   // codes per 16 bytes
  const uint16_t* row = w + static_cast<int64_t>(blockIdx.x) * K;
  float m = 0.0f;
  for (int ch = threadIdx.x; ch < (K >> 3); ch += kRtnThreads) {
    const uint4 p = *reinterpret_cast<const uint4*>(row + (ch << 3));
    m = fmaxf(m, fmaxf(fmaxf(fabsf(bf16_lo(p.x)), fabsf(bf16_hi(p.x))), fmaxf(fabsf(bf16_lo(p.y)), fabsf(bf16_hi(p.y)))));
    m = fmaxf(m, fmaxf(fmaxf(fabsf(bf16_lo(p.z)), fabsf(bf16_hi(p.z))), fmaxf(fabsf(bf16_lo(p.w)), fabsf(bf16_hi(p.w)))));
  }
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = m;
  __syncthreads();
  m = s_max[0];
#pragma unroll
  for (int i = 1; i < kRtnThreads / kWave; ++i) m = fmaxf(m, s_max[i]);
  const float s = fmaxf(m, kEps) / qmax;
  if (threadIdx.x == 0) scales[blockIdx.x] = s;
  unsigned char* orow = packed + static_cast<int64_t>(blockIdx.x) * (static_cast<int64_t>(K) * BITS / 8);
  for (int blk = threadIdx.x; blk < K / PER; blk += kRtnThreads) {
    uint32_t word[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int p = blk * PER + i;
      float q = rintf(bf16_to_f32(row[rtn_channel_of<BITS>(p)]) / s);
      q = fminf(fmaxf(q, -qmax), qmax);
      const uint32_t code = static_cast<uint32_t>(static_cast<int>(q)) & (BITS == 8 ? 0xFFu : 0xFu);
      word[(i * BITS) >> 5] |= code << ((i * BITS) & 31);
    }
    *reinterpret_cast<uint4*>(orow + blk * 16) = make_uint4(word[0], word[1], word[2], word[3]);
  }
}

hipError_t launch_rtn_pack(const uint16_t* w, int64_t n_out, int64_t n_in, int bits, void* packed, float* scales,
                           hipStream_t stream) {
  if (bits == 8)
    rtn_pack_kernel<8><<<static_cast<unsigned>(n_out), kRtnThreads, 0, stream>>>(w, static_cast<int>(n_in), static_cast<unsigned char*>(packed), scales);
  else
    rtn_pack_kernel<4><<<static_cast<unsigned>(n_out), kRtnThreads, 0, stream>>>(w, static_cast<int>(n_in), static_cast<unsigned char*>(packed), scales);
  return hipGetLastError();
}

// packed codes -> bf16 [N, K] row-major holding the integers q themselves (|q| <= 127: exact in
// bf16), channels back in natural order.  One thread per 16 packed bytes.
template <int BITS>
__global__ __launch_bounds__(256) void rtn_dequant_kernel(const unsigned char* __restrict__ packed, int64_t n_blocks,
                                                          int K, uint16_t* __restrict__ out) {
  constexpr int PER = BITS == 8 ? 16 : 32;
  const int64_t b = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (b >= n_blocks) return;
  const int blocks_per_row = K / PER;
  const int64_t n = b / blocks_per_row;
  const int blk = static_cast<int>(b - n * blocks_per_row);
  const uint4 raw = *reinterpret_cast<const uint4*>(packed + b * 16);
  const uint32_t word[4] = {raw.x, raw.y, raw.z, raw.w};
  uint16_t* orow = out + n * K;
  // positions 8m .. 8m+7 of a row are eight consecutive channels: one 16-byte store each
#pragma unroll
  for (int m = 0; m < PER / 8; ++m) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int idx = m * 8 + i;
      const int code = static_cast<int>(word[(idx * BITS) >> 5] << (32 - BITS - ((idx * BITS) & 31))) >> (32 - BITS);   // sign-extending field extract
      v[i] = static_cast<float>(code);
    }
    uint4 ob;
    ob.x = cvt_pk_bf16(v[0], v[1]); ob.y = cvt_pk_bf16(v[2], v[3]);
    ob.z = cvt_pk_bf16(v[4], v[5]); ob.w = cvt_pk_bf16(v[6], v[7]);
    *reinterpret_cast<uint4*>(orow + rtn_channel_of<BITS>(blk * PER + m * 8)) = ob;
  }
}

hipError_t launch_rtn_dequant(const void* packed, int64_t n_out, int64_t n_in, int bits, uint16_t* out, hipStream_t stream) {
  const int64_t n_blocks = n_out * n_in * bits / 8 / 16;
  const unsigned grid = static_cast<unsigned>((n_blocks + 255) / 256);
  if (bits == 8)
    rtn_dequant_kernel<8><<<grid, 256, 0, stream>>>(static_cast<const unsigned char*>(packed), n_blocks, static_cast<int>(n_in), out);
  else
    rtn_dequant_kernel<4><<<grid, 256, 0, stream>>>(static_cast<const unsigned char*>(packed), n_blocks, static_cast<int>(n_in), out);
  return hipGetLastError();
}

}  // namespace mote
