// Spatial ResBlock operator group (GroupNorm, SiLU, 3x3 convolution) for bf16 features.  The
// convolution operands (normalised activations, bounded by construction, and the kernels) are held
// as fp16: the matrix cores run fp16 and bf16 at the same rate, and fp16's three extra significand
// bits keep the operand rounding of two chained 9*C-term contractions well inside the error budget
// that the final bf16 rounding of x + branch leaves.  bf16 kernels convert exactly unless a value
// lies outside fp16's normal range (|w| < 6.1e-5 rounds to a multiple of 2^-24, |w| > 65504 overflows).
//   conv3x3_f16_kernel     3x3 convolution (zero padding 1, stride 1) as an implicit GEMM on the
//                           matrix cores over a token-major activation [M, C]               [MFMA bound]
//   pack_conv_kernel        [O, C, 3, 3] bf16 kernel -> fp16 [O, 9*C] with k = tap*C + c (k contiguous)
//   temb_proj_kernel        e[b, o] = b_t[o] + sum_k SiLU(temb[b, k]) * W_t[k, o]
//   gn_stats_tokens_kernel  GroupNorm statistics of a token-major fp32 feature per (image, group)
//   gn_silu_tokens_kernel   SiLU(GroupNorm(h)) -> fp16 operand, token-major                  [HBM bound]
#pragma once
#include "si_common.h"
#include "k_gemm.h"

namespace si {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float silu(float v) { return v / (1.f + __expf(-v)); }

// acc[m, o] = sum_{tap, c} A[m + dy*W + dx, c] * Wp[o, tap*C + c] over the taps whose source pixel
// lies inside the image (tap = 3*(dy+1) + (dx+1)); token m = img*H*W + y*W + x, A row stride C.
// Same block structure as gemm_bf16_kernel (weights as the MFMA row operand, tokens as columns, so a
// lane holds 4 consecutive output channels of one token); the activation loader shifts its rows by
// the tap's offset and zero-fills rows that fall outside the image.  C % BK == 0.
template <int BM, int BN, int WAVES_M, int WAVES_N, class Epi, int BK>
__global__ __launch_bounds__(256) void conv3x3_f16_kernel(const _Float16* __restrict__ A, const _Float16* __restrict__ Wp,
                                                           int64_t M, int C, int O, int H, int W, Epi epi) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per block");
  constexpr int LDK = BK + 8, CPR = BK / 8;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_CHUNKS = BM * CPR / 256, W_CHUNKS = (BN * CPR + 255) / 256;
  static_assert(WM % 32 == 0 && WN % 32 == 0 && A_CHUNKS >= 1, "tile shape");

  __shared__ __attribute__((aligned(16))) unsigned short As[2][BM][LDK];
  __shared__ __attribute__((aligned(16))) unsigned short Ws[2][BN][LDK];

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;
  const int K = 9 * C;
  const int P = H * W;

  // pixel coordinates of the rows this thread stages (fixed over the k loop)
  int py[A_CHUNKS], px[A_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int row = (tid + i * 256) / CPR;
    const int64_t m = m0 + row;
    const int p = (int)(m % P);
    py[i] = m < M ? p / W : -4;   // -4: no tap is ever inside
    px[i] = p % W;
  }

  uint4 ra[A_CHUNKS], rw[W_CHUNKS];
  auto load_tile = [&](int tap, int c0) {
    const int dy = tap / 3 - 1, dx = tap % 3 - 1;
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      const int id = tid + i * 256, row = id / CPR, kc = (id % CPR) * 8;
      const bool in = (unsigned)(py[i] + dy) < (unsigned)H && (unsigned)(px[i] + dx) < (unsigned)W;
      const int64_t src = m0 + row + dy * W + dx;
      ra[i] = in ? *reinterpret_cast<const uint4*>(A + src * C + c0 + kc) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      const int id = tid + i * 256, row = id / CPR, kc = (id % CPR) * 8;
      const int n = n0 + row;
      rw[i] = (row < BN && n < O) ? *reinterpret_cast<const uint4*>(Wp + (int64_t)n * K + tap * C + c0 + kc)
                                  : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      const int id = tid + i * 256, row = id / CPR, kc = (id % CPR) * 8;
      *reinterpret_cast<uint4*>(&As[buf][row][kc]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      const int id = tid + i * 256, row = id / CPR, kc = (id % CPR) * 8;
      if (row < BN) *reinterpret_cast<uint4*>(&Ws[buf][row][kc]) = rw[i];
    }
  };

  f32x16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int per_tap = C / BK, nk = 9 * per_tap;
  int tap = 0, c0 = 0;  // of the tile being loaded
  auto advance = [&]() {
    c0 += BK;
    if (c0 == C) {
      c0 = 0;
      ++tap;
    }
  };
  load_tile(tap, c0);
  advance();
  store_tile(0);
  __syncthreads();
  const int frow = lane % 32, fk = (lane / 32) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      load_tile(tap, c0);
      advance();
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      f16x8_t wf[TN], af[TM];
#pragma unroll
      for (int i = 0; i < TN; ++i) wf[i] = *reinterpret_cast<const f16x8_t*>(&Ws[cur][wn0 + i * 32 + frow][kk + fk]);
#pragma unroll
      for (int j = 0; j < TM; ++j) af[j] = *reinterpret_cast<const f16x8_t*>(&As[cur][wm0 + j * 32 + frow][kk + fk]);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[i], af[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tile(cur ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int64_t m = m0 + wm0 + j * 32 + frow;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn0 + i * 32 + q * 8 + (lane / 32) * 4;
        if (n < O) {
          const float v[4] = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
          epi(m, n, v);
        }
      }
    }
  }
}

// h[m, n] = acc + bias[n] + e[b(m), n]   (fp32, token-major; e may be NULL); b(m) = m / tokens_per_batch
struct EpiConvEmb {
  float* h;
  int64_t ld;
  const bf16* bias;
  const float* e;
  int64_t tokens_per_batch;
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    const float* er = e ? e + (m / tokens_per_batch) * ld + n0 : nullptr;
    float4 o;
    o.x = v[0] + param_or(bias, n0 + 0, 0.f) + (er ? er[0] : 0.f);
    o.y = v[1] + param_or(bias, n0 + 1, 0.f) + (er ? er[1] : 0.f);
    o.z = v[2] + param_or(bias, n0 + 2, 0.f) + (er ? er[2] : 0.f);
    o.w = v[3] + param_or(bias, n0 + 3, 0.f) + (er ? er[3] : 0.f);
    *reinterpret_cast<float4*>(h + m * ld + n0) = o;
  }
};

// dst[o, tap*C + c] = src[o, c, tap]  (src in [O, C, 3, 3] order)
__global__ __launch_bounds__(256) void pack_conv_kernel(const bf16* __restrict__ src, _Float16* __restrict__ dst, int O, int C) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)O * 9 * C;
  if (idx >= total) return;
  const int c = (int)(idx % C);
  const int tap = (int)((idx / C) % 9);
  const int64_t o = idx / ((int64_t)9 * C);
  dst[idx] = (_Float16)to_float(src[(o * C + c) * 9 + tap]);
}

// e[b, o] = b_t[o] + sum_k SiLU(temb[b, k]) * W_t[k, o]; one thread per (b, o), fp32 accumulation in k order
__global__ __launch_bounds__(256) void temb_proj_kernel(const bf16* __restrict__ temb, const bf16* __restrict__ wt,
                                                        const bf16* __restrict__ bt, float* __restrict__ e, int Kt, int O) {
  const int o = blockIdx.x * 256 + threadIdx.x;
  const int b = blockIdx.y;
  if (o >= O) return;
  float s = 0.f;
  for (int k = 0; k < Kt; ++k) s = fmaf(silu(to_float(temb[(int64_t)b * Kt + k])), to_float(wt[(int64_t)k * O + o]), s);
  e[(int64_t)b * O + o] = s + param_or(bt, o, 0.f);
}

// Statistics per (image, group) of h[img*P + p, g*ng .. (g+1)*ng): one block per (image, group);
// sums relative to the first element, fp32 lanes merged in fp64.  stats[(img*G + g)*2 + {0,1}] =
// {mean, 1/sqrt(var + eps)}.
__global__ __launch_bounds__(256) void gn_stats_tokens_kernel(const float* __restrict__ h, float* __restrict__ stats, int P,
                                                              int C, int G, float eps) {
  const int g = blockIdx.x % G, img = blockIdx.x / G;
  const int ng = C / G;
  const float* base = h + (int64_t)img * P * C + g * ng;
  const float shift = base[0];
  float s1 = 0.f, s2 = 0.f;
  for (int p = threadIdx.x; p < P; p += 256) {
    const float* r = base + (int64_t)p * C;
    for (int c = 0; c < ng; ++c) {
      const float d = r[c] - shift;
      s1 += d;
      s2 += d * d;
    }
  }
  const double a1 = wave_sum((double)s1), a2 = wave_sum((double)s2);
  __shared__ double sh[2][4];
  if (threadIdx.x % kWave == 0) {
    sh[0][threadIdx.x / kWave] = a1;
    sh[1][threadIdx.x / kWave] = a2;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const double n = (double)ng * (double)P;
    const double m1 = (sh[0][0] + sh[0][1] + sh[0][2] + sh[0][3]) / n;
    const double m2 = (sh[1][0] + sh[1][1] + sh[1][2] + sh[1][3]) / n;
    double var = m2 - m1 * m1;
    if (var < 0.0) var = 0.0;
    stats[(int64_t)blockIdx.x * 2 + 0] = (float)((double)shift + m1);
    stats[(int64_t)blockIdx.x * 2 + 1] = (float)(1.0 / sqrt(var + (double)eps));
  }
}

// a[m, c] = fp16(SiLU((h[m, c] - mean) * rstd * gamma[c] + beta[c])), four channels per thread (C % 4 == 0)
__global__ __launch_bounds__(256) void gn_silu_tokens_kernel(const float* __restrict__ h, const float* __restrict__ stats,
                                                             const bf16* __restrict__ gamma, const bf16* __restrict__ beta,
                                                             _Float16* __restrict__ a, int64_t M, int P, int C, int G) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int cv = C / 4;
  if (idx >= M * cv) return;
  const int64_t m = idx / cv;
  const int c = (int)(idx % cv) * 4;
  const int64_t img = m / P;
  const int ng = C / G;
  const float4 v = *reinterpret_cast<const float4*>(h + m * C + c);
  const float in[4] = {v.x, v.y, v.z, v.w};
  float o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int g = (c + i) / ng;
    const float mean = stats[(img * G + g) * 2 + 0], rstd = stats[(img * G + g) * 2 + 1];
    o[i] = silu((in[i] - mean) * rstd * param_or(gamma, c + i, 1.f) + param_or(beta, c + i, 0.f));
  }
  typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
  f16x4_t pk = {(_Float16)o[0], (_Float16)o[1], (_Float16)o[2], (_Float16)o[3]};
  *reinterpret_cast<f16x4_t*>(a + m * C + c) = pk;
}

}  // namespace si
