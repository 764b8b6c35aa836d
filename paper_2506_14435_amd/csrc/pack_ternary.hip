// Q_w (absmean ternary quantiser, Eq.7, Eq.9, Eq.10 of Section 3.1) and the 2-bit pack.
//
// Three launches on the caller's stream:
//   1. abs_sum_kernel   : fixed grid, each block writes one fp64 partial of sum|W| into the
//                         (not yet used) packed buffer -- deterministic, no atomics
//   2. alpha_kernel     : one block folds the partials in a fixed order, writes
//                         alpha = max(fp32(sum / (N*K)), 1e-5)
//   3. pack_kernel      : one thread per packed 32-bit word: 16 x (W / alpha -> RNE -> clip)
//                         -> code t+1 at bit 8*(i%4) + 2*(i/4)
#include "common.h"
#include "launch.h"

namespace mote {

template <typename T>
__device__ __forceinline__ float load_w(const T* w, int64_t i);
template <>
__device__ __forceinline__ float load_w<float>(const float* w, int64_t i) { return w[i]; }
template <>
__device__ __forceinline__ float load_w<uint16_t>(const uint16_t* w, int64_t i) { return bf16_to_f32(w[i]); }

constexpr int kPackThreads = 256;

template <typename T>
__global__ __launch_bounds__(kPackThreads) void abs_sum_kernel(const T* __restrict__ w, int64_t n,
                                                               double* __restrict__ partial) {
  __shared__ double s_part[kPackThreads / kWave];
  double acc = 0.0;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kPackThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kPackThreads + threadIdx.x; i < n; i += stride)
    acc += static_cast<double>(fabsf(load_w<T>(w, i)));
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kPackThreads / kWave; ++i) t += s_part[i];
    partial[blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(kPackThreads) void alpha_kernel(const double* __restrict__ partial, int n_partial,
                                                            double count, float* __restrict__ alpha) {
  __shared__ double s_part[kPackThreads / kWave];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += kPackThreads) acc += partial[i];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kPackThreads / kWave; ++i) t += s_part[i];
    const float a = static_cast<float>(t / count);
    alpha[0] = fmaxf(a, kEps);
  }
}

template <typename T>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(const T* __restrict__ w, int64_t n_words, int tiles_k,
                                                            int64_t n_in, const float* __restrict__ alpha_ptr,
                                                            bool binary, uint32_t* __restrict__ packed) {
  const int64_t wi = static_cast<int64_t>(blockIdx.x) * kPackThreads + threadIdx.x;
  if (wi >= n_words) return;
  const float alpha = alpha_ptr[0];
  const int64_t tile = wi >> 8;
  const int within = static_cast<int>(wi & 255);
  const int lane = within >> 2, s = within & 3;
  const int r = lane & 31, g = lane >> 5;
  const int64_t nt = tile / tiles_k;
  const int kt = static_cast<int>(tile - nt * tiles_k);
  const int64_t base = (nt * 32 + r) * n_in + kt * 128 + s * 32 + g * 16;
  uint32_t word = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float wv = load_w<T>(w, base + i);
    float q = rintf(wv / alpha);   // IEEE divide, round half to even
    q = fminf(fmaxf(q, -1.0f), 1.0f);
    if (binary) q = wv < 0.0f ? -1.0f : 1.0f;   // 1-bit quantiser of the routed-expert ablation: sign(w), sign(0) = +1
    const uint32_t code = static_cast<uint32_t>(static_cast<int>(q) + 1);
    word |= code << (8 * (i & 3) + 2 * (i >> 2));
  }
  packed[wi] = word;
}

template <typename T>
static hipError_t pack_impl(const T* w, int64_t n_out, int64_t n_in, uint32_t* packed, float* alpha, bool binary,
                            hipStream_t stream) {
  const int64_t n = n_out * n_in;
  const int64_t n_words = n / 16;
  // The packed buffer holds n/4 bytes >= 1024, i.e. room for >= 128 fp64 partials.
  int64_t max_partials = (n / 4) / 8;
  int64_t want = (n + kPackThreads * 16 - 1) / (kPackThreads * 16);
  int n_partial = static_cast<int>(want < 1024 ? want : 1024);
  if (n_partial > max_partials) n_partial = static_cast<int>(max_partials);
  double* partial = reinterpret_cast<double*>(packed);
  abs_sum_kernel<T><<<n_partial, kPackThreads, 0, stream>>>(w, n, partial);
  alpha_kernel<<<1, kPackThreads, 0, stream>>>(partial, n_partial, static_cast<double>(n), alpha);
  const int64_t blocks = (n_words + kPackThreads - 1) / kPackThreads;
  pack_kernel<T><<<static_cast<unsigned>(blocks), kPackThreads, 0, stream>>>(
      w, n_words, static_cast<int>(n_in / 128), n_in, alpha, binary, packed);
  return hipGetLastError();
}

hipError_t launch_pack_ternary(const void* w, bool is_bf16, int64_t n_out, int64_t n_in, uint32_t* packed,
                               float* alpha, bool binary, hipStream_t stream) {
  if (is_bf16) return pack_impl<uint16_t>(static_cast<const uint16_t*>(w), n_out, n_in, packed, alpha, binary, stream);
  return pack_impl<float>(static_cast<const float*>(w), n_out, n_in, packed, alpha, binary, stream);
}

}  // namespace mote
