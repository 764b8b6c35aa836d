// Row quantiser Q_a(h) (Eq.8-10 applied to the hidden activation of Eq.5), the weighted
// combine of Eq.2 + Eq.4, and the calibration copy kernel.
#include <stdlib.h>
#include "common.h"
#include "launch.h"

namespace mote {

constexpr int kRowThreads = 256;

template <int THREADS>
__device__ __forceinline__ float block_max(float v, float* s_buf) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) s_buf[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = s_buf[0];
#pragma unroll
  for (int i = 1; i < THREADS / kWave; ++i) r = fmaxf(r, s_buf[i]);
  __syncthreads();
  return r;
}

template <int THREADS>
__device__ __forceinline__ int block_sum(int v, int* s_buf) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) s_buf[threadIdx.x >> 6] = v;
  __syncthreads();
  int r = 0;
#pragma unroll
  for (int i = 0; i < THREADS / kWave; ++i) r += s_buf[i];
  __syncthreads();
  return r;
}

// One workgroup per dispatch row.  Rows of up to kRowThreads * kRowChunks 8-element chunks are
// read once: every thread requests all its chunks before it looks at the first (the loads are in
// flight together), takes the absmax, and quantises out of registers.  Longer rows take a second
// sweep (L2 hits) for the part that did not fit.
constexpr int kRowChunks = 6;

__device__ __forceinline__ float chunk_absmax(const uint4& p) {
  return fmaxf(fmaxf(fmaxf(fabsf(bf16_lo(p.x)), fabsf(bf16_hi(p.x))), fmaxf(fabsf(bf16_lo(p.y)), fabsf(bf16_hi(p.y)))),
               fmaxf(fmaxf(fabsf(bf16_lo(p.z)), fabsf(bf16_hi(p.z))), fmaxf(fabsf(bf16_lo(p.w)), fabsf(bf16_hi(p.w)))));
}

__device__ __forceinline__ int chunk_quant(const uint4& p, float s, uint2* o) {
  const int q0 = quant_i8(bf16_lo(p.x), s), q1 = quant_i8(bf16_hi(p.x), s);
  const int q2 = quant_i8(bf16_lo(p.y), s), q3 = quant_i8(bf16_hi(p.y), s);
  const int q4 = quant_i8(bf16_lo(p.z), s), q5 = quant_i8(bf16_hi(p.z), s);
  const int q6 = quant_i8(bf16_lo(p.w), s), q7 = quant_i8(bf16_hi(p.w), s);
  o->x = (q0 & 0xFF) | ((q1 & 0xFF) << 8) | ((q2 & 0xFF) << 16) | (static_cast<uint32_t>(q3 & 0xFF) << 24);
  o->y = (q4 & 0xFF) | ((q5 & 0xFF) << 8) | ((q6 & 0xFF) << 16) | (static_cast<uint32_t>(q7 & 0xFF) << 24);
  return q0 + q1 + q2 + q3 + q4 + q5 + q6 + q7;
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void quant_rows_kernel(const uint16_t* __restrict__ h, int F,
                                                             int8_t* __restrict__ q, float* __restrict__ beta,
                                                             int32_t* __restrict__ rowsum) {
  constexpr int kRowThreads = THREADS;
  __shared__ float s_f[kRowThreads / kWave];
  __shared__ int s_i[kRowThreads / kWave];
  const int64_t row = blockIdx.x;
  const uint16_t* hp = h + row * F;
  const int n_chunks = F >> 3;
  uint4 keep[kRowChunks];
#pragma unroll
  for (int i = 0; i < kRowChunks; ++i) {
    const int ch = threadIdx.x + i * kRowThreads;
    keep[i] = ch < n_chunks ? *reinterpret_cast<const uint4*>(hp + ch * 8) : make_uint4(0u, 0u, 0u, 0u);
  }
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < kRowChunks; ++i) amax = fmaxf(amax, chunk_absmax(keep[i]));
  for (int ch = threadIdx.x + kRowChunks * kRowThreads; ch < n_chunks; ch += kRowThreads)
    amax = fmaxf(amax, chunk_absmax(*reinterpret_cast<const uint4*>(hp + ch * 8)));
  const float b = fmaxf(block_max<THREADS>(amax, s_f), kEps);
  const float s = 127.0f / b;
  int rs = 0;
#pragma unroll
  for (int i = 0; i < kRowChunks; ++i) {
    const int ch = threadIdx.x + i * kRowThreads;
    uint2 o;
    const int part = chunk_quant(keep[i], s, &o);
    if (ch < n_chunks) {
      rs += part;
      *reinterpret_cast<uint2*>(q + row * F + ch * 8) = o;
    }
  }
  for (int ch = threadIdx.x + kRowChunks * kRowThreads; ch < n_chunks; ch += kRowThreads) {
    uint2 o;
    rs += chunk_quant(*reinterpret_cast<const uint4*>(hp + ch * 8), s, &o);
    *reinterpret_cast<uint2*>(q + row * F + ch * 8) = o;
  }
  const int total = block_sum<THREADS>(rs, s_i);
  if (threadIdx.x == 0) {
    beta[row] = b;
    rowsum[row] = total;
  }
}

hipError_t launch_quant_rows(const uint16_t* h, int rows, int F, int8_t* q, float* beta, int32_t* rowsum,
                             hipStream_t stream) {
  if (rows == 0) return hipSuccess;
  // short rows: half the threads per row still read a row in one sweep, and twice as many rows are resident
  const bool narrow = knob(kKnobQuantWide) != 1;
  if (narrow && (F >> 3) <= 128 * kRowChunks) quant_rows_kernel<128><<<rows, 128, 0, stream>>>(h, F, q, beta, rowsum);
  else quant_rows_kernel<kRowThreads><<<rows, kRowThreads, 0, stream>>>(h, F, q, beta, rowsum);
  return hipGetLastError();
}

// Combine (Eq.2 + Eq.4): one thread per (token, 8 channels).
//   y_e[c] = float(D[row, c]) * ((beta_h[row] / 127) * alpha_down[e])      (ternary linear, Section 3.1)
//   out[t, c] = y_s[t, c] + sum_j p[t, j] * y_{e_j}[c]
// D and y_s may arrive as partial planes of a K split; they are added in plane order.
template <int KMAX>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  const int d = a.d, k = a.k;
  const int chunks = d >> 3;
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (gid >= static_cast<int64_t>(a.T) * chunks) return;
  const int t = static_cast<int>(gid / chunks);
  const int c0 = static_cast<int>(gid - static_cast<int64_t>(t) * chunks) << 3;
  const int64_t yo = static_cast<int64_t>(t) * d + c0;
  // Partial planes are requested four at a time (the loads of a batch are in flight together: a
  // plane-by-plane loop pays one memory round trip per plane) and added in plane order.
  float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int p0 = 0; p0 < a.y_planes; p0 += 4) {
    float4 s0[4], s1[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (p0 + u < a.y_planes) {
        s0[u] = *reinterpret_cast<const float4*>(a.y_s + (p0 + u) * a.y_stride + yo);
        s1[u] = *reinterpret_cast<const float4*>(a.y_s + (p0 + u) * a.y_stride + yo + 4);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (p0 + u < a.y_planes) {
        o[0] += s0[u].x; o[1] += s0[u].y; o[2] += s0[u].z; o[3] += s0[u].w;
        o[4] += s1[u].x; o[5] += s1[u].y; o[6] += s1[u].z; o[7] += s1[u].w;
      }
    }
  }
  if (a.tap_y_s) {
    *reinterpret_cast<float4*>(a.tap_y_s + yo) = make_float4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<float4*>(a.tap_y_s + yo + 4) = make_float4(o[4], o[5], o[6], o[7]);
  }
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    if (j < k) {
      const int row = a.row_of[t * k + j];
      const int e = a.topk_idx[t * k + j];
      const float p = a.topk_p[t * k + j];
      const float sc = (a.beta_h[row] / 127.0f) * a.alpha[e * 3 + 2];
      const int64_t ro = static_cast<int64_t>(row) * d + c0;
      int dsum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      const int d_planes = a.row_planes ? 1 + ((a.row_planes[row] >> (2 * (c0 / a.d_tile_n))) & 3) : a.d_planes;
      for (int p0 = 0; p0 < d_planes; p0 += 4) {
        int4 d0[4], d1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (p0 + u < d_planes) {
            d0[u] = *reinterpret_cast<const int4*>(a.acc_down + (p0 + u) * a.d_stride + ro);
            d1[u] = *reinterpret_cast<const int4*>(a.acc_down + (p0 + u) * a.d_stride + ro + 4);
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (p0 + u < d_planes) {
            dsum[0] += d0[u].x; dsum[1] += d0[u].y; dsum[2] += d0[u].z; dsum[3] += d0[u].w;
            dsum[4] += d1[u].x; dsum[5] += d1[u].y; dsum[6] += d1[u].z; dsum[7] += d1[u].w;
          }
        }
      }
      if (a.tap_acc_down) {
        *reinterpret_cast<int4*>(a.tap_acc_down + ro) = make_int4(dsum[0], dsum[1], dsum[2], dsum[3]);
        *reinterpret_cast<int4*>(a.tap_acc_down + ro + 4) = make_int4(dsum[4], dsum[5], dsum[6], dsum[7]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = fmaf(p, static_cast<float>(dsum[i]) * sc, o[i]);
    }
  }
  if (a.residual) {   // x^a of Eq.2, added in fp32 before the single rounding
    const uint4 rb = *reinterpret_cast<const uint4*>(a.residual + yo);
    o[0] += bf16_lo(rb.x); o[1] += bf16_hi(rb.x); o[2] += bf16_lo(rb.y); o[3] += bf16_hi(rb.y);
    o[4] += bf16_lo(rb.z); o[5] += bf16_hi(rb.z); o[6] += bf16_lo(rb.w); o[7] += bf16_hi(rb.w);
  }
  uint4 ob;
  ob.x = cvt_pk_bf16(o[0], o[1]);
  ob.y = cvt_pk_bf16(o[2], o[3]);
  ob.z = cvt_pk_bf16(o[4], o[5]);
  ob.w = cvt_pk_bf16(o[6], o[7]);
  *reinterpret_cast<uint4*>(a.out + yo) = ob;
  if (a.out_f32) {
    *reinterpret_cast<float4*>(a.out_f32 + yo) = make_float4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<float4*>(a.out_f32 + yo + 4) = make_float4(o[4], o[5], o[6], o[7]);
  }
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t stream) {
  if (a.T == 0) return hipSuccess;
  const int64_t n = static_cast<int64_t>(a.T) * (a.d >> 3);
  const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
  combine_kernel<8><<<blocks, 256, 0, stream>>>(a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = static_cast<size_t>(gridDim.x) * 256;
  for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t stream) {
  const size_t n16 = n_bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  copy_kernel<<<static_cast<unsigned>(blocks), 256, 0, stream>>>(static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
  return hipGetLastError();
}

}  // namespace mote
