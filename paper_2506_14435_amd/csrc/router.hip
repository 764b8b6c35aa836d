// Router (gate softmax of Eq.3 + GShard-style top-k, Section 3.1) fused with the
// per-token absmax int8 quantiser Q_a(x) (Eq.8-10), and the dispatch plan that turns the
// top-k indices into an expert-major row permutation.
//
// router_quant_kernel: one workgroup owns TPW tokens, its four wavefronts split the channels.
// Each lane owns 8-channel chunks of the token rows (16-byte bf16 loads), multiplies them with the matching 8 rows of the
// bf16 router matrix and accumulates TPW x EMAX partial logits in fp64 (a bf16 x bf16
// product is exact, and fp64 accumulation makes the selected indices independent of the
// summation order).  A 6-step butterfly reduce-scatter leaves lane l with the finished
// logit (token l / EMAX, expert l % EMAX).  The token rows are then read a second time
// (L2 hits) to emit the int8 row, its absmax and its integer row sum.
#include "common.h"
#include "launch.h"

namespace mote {


template <int OFF, int N>
__device__ __forceinline__ void reduce_scatter_step(double (&v)[N], int lane) {
  constexpr int kHalf = OFF;  // values kept after this step == OFF (64 -> 32 -> ... -> 1)
  const bool up = (lane & OFF) != 0;
#pragma unroll
  for (int i = 0; i < kHalf; ++i) {
    const double keep = up ? v[i + kHalf] : v[i];
    const double send = up ? v[i] : v[i + kHalf];
    v[i] = keep + __shfl_xor(send, OFF, kWave);
  }
  if constexpr (OFF > 1) reduce_scatter_step<OFF / 2, N>(v, lane);
}

template <int EMAX>
__device__ __forceinline__ void load_router_row(const uint16_t* __restrict__ row, int E, bool vec_ok,
                                                double (&w)[EMAX]) {
  if (vec_ok) {
#pragma unroll
    for (int v = 0; v < EMAX / 8; ++v) {
      if (v * 8 < E) {
        const uint4 p = *reinterpret_cast<const uint4*>(row + v * 8);
        w[v * 8 + 0] = bf16_lo(p.x); w[v * 8 + 1] = bf16_hi(p.x);
        w[v * 8 + 2] = bf16_lo(p.y); w[v * 8 + 3] = bf16_hi(p.y);
        w[v * 8 + 4] = bf16_lo(p.z); w[v * 8 + 5] = bf16_hi(p.z);
        w[v * 8 + 6] = bf16_lo(p.w); w[v * 8 + 7] = bf16_hi(p.w);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) w[v * 8 + j] = 0.0;
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < EMAX; ++e) w[e] = (e < E) ? static_cast<double>(bf16_to_f32(row[e])) : 0.0;
  }
}

// Gate softmax (Eq.3) and top-k of one token on the EMAX consecutive lanes that hold its logits
// (lane's expert e; logits beyond E are padding).  `store`: whether this lane group's token exists
// and is this group's to write (the lanes still take part in the shuffles otherwise).
template <int EMAX>
__device__ __forceinline__ void gate_topk(double l, int e, bool store, int tok, const float* __restrict__ bias, int E,
                                          int k, int32_t* __restrict__ topk_idx, float* __restrict__ topk_p,
                                          float* __restrict__ gate_p) {
  const bool valid = e < E;
  if (bias != nullptr && valid) l += static_cast<double>(bias[e]);
  // A non-finite hidden state must not be able to select a padding lane: NaN and -inf logits
  // are ranked as the lowest finite value, still above the padding (-1e300) and the taken
  // (-1.7e300) lanes, so the k winners are always experts below E.
  if (!(l > -1.0e299)) l = -1.0e299;
  if (!valid) l = -1.0e300;
  // gate softmax (Eq.3) over the EMAX lanes of a token: max and sum by xor shuffles
  double mx = l;
#pragma unroll
  for (int off = EMAX / 2; off > 0; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off, kWave));
  // fp64 like the logits; P is rounded to fp32 once
  const double ex = valid ? exp(l - mx) : 0.0;
  double sum = ex;
#pragma unroll
  for (int off = EMAX / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
  const float pr = static_cast<float>(ex / sum);
  if (gate_p != nullptr && valid && store)
    gate_p[static_cast<int64_t>(tok) * E + e] = pr;   // the whole gate distribution (Eq.12 needs it)
  // top-k: k rounds of an arg-max butterfly over the EMAX lanes of a token.  Every lane of the
  // group ends a round with the winner (largest logit, ties to the lower expert index); the
  // winner's own lane then leaves the contest.
  double cur = l;                      // invalid experts sit at -1e300, taken ones go below that
  for (int j = 0; j < k; ++j) {
    double bl = cur;
    int be = e;
    float bp = pr;
#pragma unroll
    for (int off = EMAX / 2; off > 0; off >>= 1) {
      const double ol = __shfl_xor(bl, off, kWave);
      const int oe = __shfl_xor(be, off, kWave);
      const float op = __shfl_xor(bp, off, kWave);
      const bool take = (ol > bl) || (ol == bl && oe < be);
      bl = take ? ol : bl;
      be = take ? oe : be;
      bp = take ? op : bp;
    }
    if (be == e) cur = -1.7e300;
    if (e == 0 && store) {
      topk_idx[static_cast<int64_t>(tok) * k + j] = be;
      topk_p[static_cast<int64_t>(tok) * k + j] = bp;
    }
  }
}

template <int EMAX, int TPW, int NW>
__global__ __launch_bounds__(64 * NW) void router_quant_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router, const float* __restrict__ bias, int T,
    int d, int E, int k, int32_t* __restrict__ topk_idx, float* __restrict__ topk_p, int8_t* __restrict__ q_x,
    float* __restrict__ beta_x, int32_t* __restrict__ rowsum_x, float* __restrict__ gate_p) {
  constexpr int NV = EMAX * TPW;           // logits of a token group; lane l ends up with logit l % NV
  static_assert(NV <= 64 && 64 % NV == 0, "at most one finished logit per lane");
  constexpr int kWaves = NW;               // wavefronts that split the channels of one token group
  constexpr int kThreads = 64 * NW;
  __shared__ double s_logit[kWaves][64];
  __shared__ float s_amax[kWaves][TPW];
  __shared__ int s_rsum[kWaves][TPW];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * TPW;   // the NW wavefronts of a workgroup split the channels of TPW tokens
  if (t0 >= T) return;
  const int n_chunks = d >> 3;
  const bool vec_ok = (E & 7) == 0;

  const uint16_t* xrow[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) xrow[t] = x + static_cast<int64_t>(min(t0 + t, T - 1)) * d;

  double acc[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) acc[i] = 0.0;
  float amax[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) amax[t] = 0.0f;

  // with at most one chunk per lane the token values stay in registers for the quantisation pass
  const bool single_pass = n_chunks <= kThreads;
  u4 xkeep[TPW];   // plain register vectors
#pragma unroll
  for (int t = 0; t < TPW; ++t) xkeep[t] = u4{0u, 0u, 0u, 0u};
  for (int ch = wave * kWave + lane; ch < n_chunks; ch += kThreads) {
    const int c0 = ch << 3;
    float xf[TPW][8];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const uint4 p = *reinterpret_cast<const uint4*>(xrow[t] + c0);
      xkeep[t] = u4{p.x, p.y, p.z, p.w};
      xf[t][0] = bf16_lo(p.x); xf[t][1] = bf16_hi(p.x); xf[t][2] = bf16_lo(p.y); xf[t][3] = bf16_hi(p.y);
      xf[t][4] = bf16_lo(p.z); xf[t][5] = bf16_hi(p.z); xf[t][6] = bf16_lo(p.w); xf[t][7] = bf16_hi(p.w);
#pragma unroll
      for (int i = 0; i < 8; ++i) amax[t] = fmaxf(amax[t], fabsf(xf[t][i]));
    }
    constexpr int kRowUnroll = EMAX > 16 ? 1 : 2;
#pragma unroll kRowUnroll
    for (int i = 0; i < 8; ++i) {
      double w[EMAX];
      load_router_row<EMAX>(w_router + static_cast<int64_t>(c0 + i) * E, E, vec_ok, w);
#pragma unroll
      for (int t = 0; t < TPW; ++t) {
        const double xv = static_cast<double>(xf[t][i]);
#pragma unroll
        for (int e = 0; e < EMAX; ++e) acc[t * EMAX + e] = fma(xv, w[e], acc[t * EMAX + e]);
      }
    }
  }

  // lane l holds this wavefront's share of logit(token (l % NV) / EMAX, expert l % EMAX): reduce-scatter
  // over the low lane bits, then (fewer than 64 logits) a butterfly sum over the remaining ones
  if constexpr (NV > 1) reduce_scatter_step<NV / 2, NV>(acc, lane);
#pragma unroll
  for (int off = NV; off < 64; off <<= 1) acc[0] += __shfl_xor(acc[0], off, kWave);
  s_logit[wave][lane] = acc[0];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    amax[t] = wave_max(amax[t]);
    if (lane == 0) s_amax[wave][t] = amax[t];
  }
  __syncthreads();
  if (wave == 0) {   // fixed summation order over the channel slices
    double l = s_logit[0][lane];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) l += s_logit[w][lane];
    const int e = lane % EMAX;
    const int tok = t0 + (lane % NV) / EMAX;
    gate_topk<EMAX>(l, e, lane < NV && tok < T, tok, bias, E, k, topk_idx, topk_p, gate_p);
  }
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    float m = s_amax[0][t];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, s_amax[w][t]);
    amax[t] = m;
  }

  if (q_x == nullptr) return;
  // Q_a(x): beta = max(absmax, 1e-5); s = 127 / beta (IEEE divide); q = clip(rne(x * s)).
  float scale[TPW];
  int rs[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    amax[t] = fmaxf(amax[t], kEps);
    scale[t] = 127.0f / amax[t];
    rs[t] = 0;
  }
  for (int ch = wave * kWave + lane; ch < n_chunks; ch += kThreads) {
    const int c0 = ch << 3;
    // all token rows are in registers before the first store: a wait for a load would otherwise
    // also wait for the stores issued before it (one counter for both)
    u4 px[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) px[t] = single_pass ? xkeep[t] : *reinterpret_cast<const u4*>(xrow[t] + c0);
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const u4 p = px[t];
      const int q0 = quant_i8(bf16_lo(p.x), scale[t]), q1 = quant_i8(bf16_hi(p.x), scale[t]);
      const int q2 = quant_i8(bf16_lo(p.y), scale[t]), q3 = quant_i8(bf16_hi(p.y), scale[t]);
      const int q4 = quant_i8(bf16_lo(p.z), scale[t]), q5 = quant_i8(bf16_hi(p.z), scale[t]);
      const int q6 = quant_i8(bf16_lo(p.w), scale[t]), q7 = quant_i8(bf16_hi(p.w), scale[t]);
      rs[t] += q0 + q1 + q2 + q3 + q4 + q5 + q6 + q7;
      uint2 o;
      o.x = (q0 & 0xFF) | ((q1 & 0xFF) << 8) | ((q2 & 0xFF) << 16) | (static_cast<uint32_t>(q3 & 0xFF) << 24);
      o.y = (q4 & 0xFF) | ((q5 & 0xFF) << 8) | ((q6 & 0xFF) << 16) | (static_cast<uint32_t>(q7 & 0xFF) << 24);
      if (t0 + t < T) *reinterpret_cast<uint2*>(q_x + static_cast<int64_t>(t0 + t) * d + c0) = o;
    }
  }
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int part = wave_sum(rs[t]);
    if (lane == 0) s_rsum[wave][t] = part;
  }
  __syncthreads();
  if (threadIdx.x < TPW && t0 + threadIdx.x < T) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) total += s_rsum[w][threadIdx.x];
    float m = s_amax[0][threadIdx.x];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, s_amax[w][threadIdx.x]);
    beta_x[t0 + threadIdx.x] = fmaxf(m, kEps);
    rowsum_x[t0 + threadIdx.x] = total;
  }
}

// ------------------------------------------------------------------------ many tokens, E <= 16
// The logits of 16 tokens x 16 experts are one accumulator tile of the fp64 matrix instruction
// (v_mfma_f64_16x16x4: the products of bf16 values are exact in fp64, the sums are fp64 as in the
// kernel above, one instruction where that kernel issues sixteen vector FMAs).  A workgroup of four
// wavefronts owns 16 tokens; wavefront w takes the channels 128 j + 32 w .. + 31 of every 128.  Lane
// (t = lane % 16, g = lane / 16) loads the 8 channels 128 j + 32 w + 8 g .. + 7 of token t (16 bytes) for
// every j up front and keeps them in registers for the quantisation pass: element i of that chunk is
// this lane's A operand (row t, contraction slot g) of MFMA (j, i), whose B operand (slot g, expert
// lane % 16) is router row 128 j + 32 w + 8 g + i.  The router matrix goes through LDS in blocks of 256
// channels, converted to fp64 once per workgroup and stored in the order the B operands are read:
// [group (j, w)][i][lane], rows of 64 doubles padded by 16 bytes so that the staging writes (one channel
// row per thread, sixteen experts = 128 contiguous bytes) spread over the banks.
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int kRmTokens = 16;
// From this many tokens on.  Measured (d = 2048, E = 16): T = 8192 40.9 -> 30.8 us, T = 16384 at d = 3584
// 125 -> 97 us; at T <= 2048 the T / 16 workgroups are too few and the kernels above are as fast or faster
// (T = 1024: 13 vs 19 us).  Both kernels are bound by fp64 issue: one matrix instruction takes 40-60 ns per
// SIMD for its 1024 multiply-adds, about what sixteen vector FMAs take.
constexpr int kRmMinTokens = 4096;
constexpr int kRmBlockChannels = 256;
constexpr int kRmRowBytes = 64 * 8 + 16;

template <int NGW>   // upper bound of the 128-channel steps (d / 128) the registers are sized for
__global__ __launch_bounds__(256) void router_mfma_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router, const float* __restrict__ bias, int T,
    int d, int E, int k, int32_t* __restrict__ topk_idx, float* __restrict__ topk_p, int8_t* __restrict__ q_x,
    float* __restrict__ beta_x, int32_t* __restrict__ rowsum_x, float* __restrict__ gate_p) {
  __shared__ __attribute__((aligned(16))) unsigned char s_b[(kRmBlockChannels / 32) * 8 * kRmRowBytes];
  __shared__ double s_part[4][kRmTokens][16];
  __shared__ float s_amax[4][kRmTokens];
  __shared__ int s_rsum[4][kRmTokens];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = lane & 15, g = lane >> 4;
  const int t0 = blockIdx.x * kRmTokens;
  const int ngw = d >> 7;
  const uint16_t* const xrow = x + static_cast<int64_t>(min(t0 + t, T - 1)) * d + 32 * wave + 8 * g;

  u4 xk[NGW];
#pragma unroll
  for (int j = 0; j < NGW; ++j)
    xk[j] = j < ngw ? *reinterpret_cast<const u4*>(xrow + 128 * j) : u4{0u, 0u, 0u, 0u};

  v4d acc = {0.0, 0.0, 0.0, 0.0};
  float amax = 0.0f;
  // staging: thread sc owns channel row sc of the block; its router row (E bf16 values, zero beyond E) is
  // fetched one block ahead, so that it travels while the previous block is contracted
  const int sc = threadIdx.x;
  unsigned char* const s_dst = s_b + (((sc >> 5) * 8 + (sc & 7)) * kRmRowBytes) + ((sc >> 3) & 3) * 128;
  const bool vec_ok = (E & 7) == 0;
  auto load_w = [&](int jb, uint32_t (&wq)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) wq[i] = 0u;
    const int c = jb * 128 + sc;
    if (jb < ngw && c < d) {
      const uint16_t* const wr = w_router + static_cast<int64_t>(c) * E;
      if (vec_ok) {
        const u4 lo = *reinterpret_cast<const u4*>(wr);
        wq[0] = lo.x; wq[1] = lo.y; wq[2] = lo.z; wq[3] = lo.w;
        if (E > 8) {
          const u4 hi = *reinterpret_cast<const u4*>(wr + 8);
          wq[4] = hi.x; wq[5] = hi.y; wq[6] = hi.z; wq[7] = hi.w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (e < E) wq[e >> 1] |= static_cast<uint32_t>(wr[e]) << (16 * (e & 1));
      }
    }
  };
  uint32_t wq[8];
  load_w(0, wq);
#pragma unroll
  for (int jb = 0; jb < NGW; jb += 2) {   // blocks of 256 channels = two steps j
    if (jb < ngw) {
      __syncthreads();   // every wavefront is done with the previous block
#pragma unroll
      for (int e = 0; e < 16; e += 2)
        *reinterpret_cast<double2*>(s_dst + e * 8) =
            make_double2(static_cast<double>(bf16_lo(wq[e >> 1])), static_cast<double>(bf16_hi(wq[e >> 1])));
      load_w(jb + 2, wq);
      __syncthreads();
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = jb + jj;
        if (j < NGW && j < ngw) {
          const u4 p = xk[j];
          const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
          const unsigned char* const rows = s_b + (jj * 4 + wave) * 8 * kRmRowBytes + lane * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float xv = (i & 1) ? bf16_hi(pw[i >> 1]) : bf16_lo(pw[i >> 1]);
            amax = fmaxf(amax, fabsf(xv));
            const double b = *reinterpret_cast<const double*>(rows + i * kRmRowBytes);
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(static_cast<double>(xv), b, acc, 0, 0, 0);
          }
        }
      }
    }
  }

  // accumulator element v of lane (t, g) is logit (token g + 4 v, expert t) over this wavefront's channels
#pragma unroll
  for (int v = 0; v < 4; ++v) s_part[wave][g + 4 * v][t] = acc[v];
  amax = fmaxf(amax, __shfl_xor(amax, 16, kWave));
  amax = fmaxf(amax, __shfl_xor(amax, 32, kWave));
  if (g == 0) s_amax[wave][t] = amax;
  __syncthreads();
  {   // wavefront w finishes tokens 4 w .. 4 w + 3: lane = 16 * (token % 4) + expert; fixed summation order
    const int tl = 4 * wave + (lane >> 4), e = lane & 15;
    const double l = ((s_part[0][tl][e] + s_part[1][tl][e]) + s_part[2][tl][e]) + s_part[3][tl][e];
    gate_topk<16>(l, e, t0 + tl < T, t0 + tl, bias, E, k, topk_idx, topk_p, gate_p);
  }
  if (q_x == nullptr) return;
  // Q_a(x): beta = max(absmax, 1e-5); s = 127 / beta (IEEE divide); q = clip(rne(x * s)).
  const float beta = fmaxf(fmaxf(fmaxf(s_amax[0][t], s_amax[1][t]), fmaxf(s_amax[2][t], s_amax[3][t])), kEps);
  const float scale = 127.0f / beta;
  int rs = 0;
  int8_t* const qrow = q_x + static_cast<int64_t>(t0 + t) * d + 32 * wave + 8 * g;
#pragma unroll
  for (int j = 0; j < NGW; ++j) {
    if (j < ngw) {
      const u4 p = xk[j];
      const int q0 = quant_i8(bf16_lo(p.x), scale), q1 = quant_i8(bf16_hi(p.x), scale);
      const int q2 = quant_i8(bf16_lo(p.y), scale), q3 = quant_i8(bf16_hi(p.y), scale);
      const int q4 = quant_i8(bf16_lo(p.z), scale), q5 = quant_i8(bf16_hi(p.z), scale);
      const int q6 = quant_i8(bf16_lo(p.w), scale), q7 = quant_i8(bf16_hi(p.w), scale);
      rs += q0 + q1 + q2 + q3 + q4 + q5 + q6 + q7;
      uint2 o;
      o.x = (q0 & 0xFF) | ((q1 & 0xFF) << 8) | ((q2 & 0xFF) << 16) | (static_cast<uint32_t>(q3 & 0xFF) << 24);
      o.y = (q4 & 0xFF) | ((q5 & 0xFF) << 8) | ((q6 & 0xFF) << 16) | (static_cast<uint32_t>(q7 & 0xFF) << 24);
      if (t0 + t < T) *reinterpret_cast<uint2*>(qrow + 128 * j) = o;
    }
  }
  rs += __shfl_xor(rs, 16, kWave);
  rs += __shfl_xor(rs, 32, kWave);
  if (g == 0) s_rsum[wave][t] = rs;
  __syncthreads();
  if (threadIdx.x < kRmTokens && t0 + threadIdx.x < T) {
    const int tt = threadIdx.x;
    beta_x[t0 + tt] = fmaxf(fmaxf(fmaxf(s_amax[0][tt], s_amax[1][tt]), fmaxf(s_amax[2][tt], s_amax[3][tt])), kEps);
    rowsum_x[t0 + tt] = s_rsum[0][tt] + s_rsum[1][tt] + s_rsum[2][tt] + s_rsum[3][tt];
  }
}

// Up to this many tokens every token gets a workgroup of its own.
static int router_token_blocks() { return knob(kKnobRouterTokenBlocks); }

hipError_t launch_router_quant(const uint16_t* x, const uint16_t* w_router, const float* bias, int T, int d,
                               int E, int k, int32_t* topk_idx, float* topk_p, int8_t* q_x, float* beta_x,
                               int32_t* rowsum_x, float* gate_p, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  // Few tokens: four wavefronts share a token group so that more of the chip takes part;
  // many tokens: one wavefront per group keeps the cross-lane reduction cost per token low.
  const bool coop = T <= 2048;
  if (E <= 16) {
    constexpr int kTpw = 4;
    const int blocks = (T + kTpw - 1) / kTpw;
    if (T <= router_token_blocks())   // a few tokens: one token per workgroup, a quarter of the arithmetic and of the reduction per lane
      router_quant_kernel<16, 1, 4><<<T, 256, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x, beta_x,
                                                           rowsum_x, gate_p);
    else if (T >= kRmMinTokens && d <= 4096) {   // 16 tokens per workgroup on the fp64 matrix instruction
      const int wgs = (T + kRmTokens - 1) / kRmTokens;
      if (d <= 1024)
        router_mfma_kernel<8><<<wgs, 256, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x, beta_x,
                                                       rowsum_x, gate_p);
      else if (d <= 2048)
        router_mfma_kernel<16><<<wgs, 256, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x, beta_x,
                                                        rowsum_x, gate_p);
      else
        router_mfma_kernel<32><<<wgs, 256, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x, beta_x,
                                                        rowsum_x, gate_p);
    }
    else if (coop)
      router_quant_kernel<16, kTpw, 4><<<blocks, 256, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x,
                                                                   beta_x, rowsum_x, gate_p);
    else
      router_quant_kernel<16, kTpw, 1><<<blocks, 64, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x,
                                                                   beta_x, rowsum_x, gate_p);
  } else {
    if (coop)
      router_quant_kernel<64, 1, 4><<<T, 256, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x, beta_x,
                                                           rowsum_x, gate_p);
    else
      router_quant_kernel<64, 1, 1><<<T, 64, 0, stream>>>(x, w_router, bias, T, d, E, k, topk_idx, topk_p, q_x, beta_x,
                                                           rowsum_x, gate_p);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------ dispatch plan
constexpr int kPlanThreads = 1024;

// One block per expert.  Every block histograms all R = T*k indices (so it knows every
// expert's count without a grid-wide dependency), then compacts the positions of its own
// expert in ascending flat order t*k + j: the dispatch order is deterministic and stable.
__global__ __launch_bounds__(kPlanThreads) void dispatch_plan_kernel(const int32_t* __restrict__ topk_idx, int R,
                                                                     int k, int E, int tile_m, DispatchPlan plan) {
  constexpr int kItems = 4;                       // indices per thread and pass: they stay in registers
  constexpr int kPass = kItems * kPlanThreads;
  constexpr int kPlanWaves = kPlanThreads / kWave;
  __shared__ int s_cnt[64];
  __shared__ int s_wave[kItems][kPlanWaves];
  __shared__ int s_off, s_tile_base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e = blockIdx.x;
  if (tid < 64) s_cnt[tid] = 0;
  if (e == 0 && tid < 16 * kSchedStride) plan.sched[tid] = 0;
  __syncthreads();
  int first[kItems];                              // the first pass is kept for the compaction
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int i = j * kPlanThreads + tid;
    first[j] = i < R ? topk_idx[i] : -1;
  }
#pragma unroll
  for (int j = 0; j < kItems; ++j)
    if (first[j] >= 0) atomicAdd(&s_cnt[first[j]], 1);
  for (int i = kPass + tid; i < R; i += kPlanThreads) atomicAdd(&s_cnt[topk_idx[i]], 1);
  __syncthreads();
  if (tid == 0) {
    int off = 0, tiles = 0;
    for (int j = 0; j < E; ++j) {
      if (j == e) { s_off = off; s_tile_base = tiles; }
      if (e == 0) { plan.counts[j] = s_cnt[j]; plan.offsets[j] = off; }
      off += s_cnt[j];
      tiles += (s_cnt[j] + tile_m - 1) / tile_m;
    }
    if (e == 0) { plan.offsets[E] = off; plan.n_tiles[0] = tiles; }
  }
  __syncthreads();
  const int my_off = s_off, my_cnt = s_cnt[e], tile_base = s_tile_base;
  for (int m = tid; m * tile_m < my_cnt; m += kPlanThreads) {
    plan.tile_expert[tile_base + m] = e;
    plan.tile_row0[tile_base + m] = my_off + m * tile_m;
    plan.tile_rows[tile_base + m] = min(tile_m, my_cnt - m * tile_m);
  }
  // Compaction, kItems * kPlanThreads indices per pass: index j * kPlanThreads + tid of the pass is
  // item j of this thread, so (item, wavefront, lane) order is ascending flat order.
  int running = 0;
  for (int base = 0; base < R; base += kPass) {
    bool flag[kItems];
    int prefix[kItems];
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      const int i = base + j * kPlanThreads + tid;
      const int v = base == 0 ? first[j] : (i < R ? topk_idx[i] : -1);
      flag[j] = v == e;
      const uint64_t mask = __ballot(flag[j]);
      prefix[j] = __popcll(mask & ((1ull << lane) - 1ull));
      if (lane == 0) s_wave[j][wave] = __popcll(mask);
    }
    __syncthreads();
    int before[kItems], total = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      before[j] = total;
#pragma unroll
      for (int w = 0; w < kPlanWaves; ++w) {
        const int c = s_wave[j][w];
        if (w < wave) before[j] += c;
        total += c;
      }
    }
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      if (flag[j]) {
        const int i = base + j * kPlanThreads + tid;
        const int slot = my_off + running + before[j] + prefix[j];
        plan.row_of[i] = slot;
        plan.tok_of[slot] = i / k;
        plan.row_planes[slot] = 0;
      }
    }
    running += total;
    __syncthreads();
  }
}

// Histogram of the selected experts (mote_router_topk's optional output).
__global__ __launch_bounds__(kPlanThreads) void expert_counts_kernel(const int32_t* __restrict__ topk_idx, int R, int E,
                                                                     int32_t* __restrict__ counts) {
  __shared__ int s_cnt[64];
  if (threadIdx.x < 64) s_cnt[threadIdx.x] = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < R; i += kPlanThreads) atomicAdd(&s_cnt[topk_idx[i]], 1);
  __syncthreads();
  if (threadIdx.x < E) counts[threadIdx.x] = s_cnt[threadIdx.x];
}

hipError_t launch_expert_counts(const int32_t* topk_idx, int R, int E, int32_t* counts, hipStream_t stream) {
  expert_counts_kernel<<<1, kPlanThreads, 0, stream>>>(topk_idx, R, E, counts);
  return hipGetLastError();
}

hipError_t launch_dispatch_plan(const int32_t* topk_idx, int T, int k, int E, int tile_m, const DispatchPlan& plan,
                                hipStream_t stream) {
  dispatch_plan_kernel<<<E, kPlanThreads, 0, stream>>>(topk_idx, T * k, k, E, tile_m, plan);
  return hipGetLastError();
}

}  // namespace mote
