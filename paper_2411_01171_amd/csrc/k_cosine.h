// Step Rehash similarity test: cosine of two flattened features against a threshold.
//   cosine_partial_kernel  grid-stride pass over both tensors, 16-byte loads;
//                          every product is exact (bf16*bf16 in fp32, fp32*fp32
//                          in fp64) and accumulation is fp64, in a fixed order
//                          for a given n: partial[block] = {dot, |a|^2, |b|^2}.
//   cosine_finish_kernel   one block sums the partials in a fixed order, forms
//                          the cosine and takes the decision.
// HBM bound: 2 * n * sizeof(T) bytes read, 24 bytes per block written.
#pragma once
#include "si_common.h"

namespace si {

constexpr int kCosBlock = 256;
constexpr int kCosMaxBlocks = 2048;

template <typename T>
__global__ __launch_bounds__(kCosBlock) void cosine_partial_kernel(const T* __restrict__ a, const T* __restrict__ b,
                                                                   int64_t n, double* __restrict__ partial) {
  constexpr int VEC = 16 / sizeof(T);
  const int64_t nvec = n / VEC;
  const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t gstride = (int64_t)gridDim.x * blockDim.x;
  double dot = 0.0, na = 0.0, nb = 0.0;
  for (int64_t v = gtid; v < nvec; v += gstride) {
    if constexpr (sizeof(T) == 2) {
      const uint4 ra = reinterpret_cast<const uint4*>(a)[v];
      const uint4 rb = reinterpret_cast<const uint4*>(b)[v];
      const unsigned wa[4] = {ra.x, ra.y, ra.z, ra.w}, wb[4] = {rb.x, rb.y, rb.z, rb.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a0 = __uint_as_float(wa[i] << 16), a1 = __uint_as_float(wa[i] & 0xffff0000u);
        const float b0 = __uint_as_float(wb[i] << 16), b1 = __uint_as_float(wb[i] & 0xffff0000u);
        // 8-bit significands: each product is exact in fp32
        dot += (double)(a0 * b0);
        dot += (double)(a1 * b1);
        na += (double)(a0 * a0);
        na += (double)(a1 * a1);
        nb += (double)(b0 * b0);
        nb += (double)(b1 * b1);
      }
    } else {
      const float4 ra = reinterpret_cast<const float4*>(a)[v];
      const float4 rb = reinterpret_cast<const float4*>(b)[v];
      const float fa[4] = {ra.x, ra.y, ra.z, ra.w}, fb[4] = {rb.x, rb.y, rb.z, rb.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const double da = fa[i], db = fb[i];
        dot = fma(da, db, dot);
        na = fma(da, da, na);
        nb = fma(db, db, nb);
      }
    }
  }
  // ragged tail: fewer than VEC elements, one per thread of the first block
  const int64_t tail0 = nvec * VEC;
  if (blockIdx.x == 0 && tail0 + threadIdx.x < n) {
    const double da = to_float(a[tail0 + threadIdx.x]), db = to_float(b[tail0 + threadIdx.x]);
    dot = fma(da, db, dot);
    na = fma(da, da, na);
    nb = fma(db, db, nb);
  }
  dot = wave_sum(dot);
  na = wave_sum(na);
  nb = wave_sum(nb);
  __shared__ double sh[3][kCosBlock / kWave];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (lane == 0) {
    sh[0][wave] = dot;
    sh[1][wave] = na;
    sh[2][wave] = nb;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kCosBlock / kWave; ++w) s += sh[threadIdx.x][w];
    partial[(int64_t)blockIdx.x * 3 + threadIdx.x] = s;
  }
}

// result layout: cos (double) at result_cos (nullable), decision (int32) at result_dec.
__global__ __launch_bounds__(kCosBlock) void cosine_finish_kernel(const double* __restrict__ partial, int nblocks, double gamma,
                                                                  double* __restrict__ result_cos, int* __restrict__ result_dec) {
  double acc[3] = {0.0, 0.0, 0.0};
  for (int i = threadIdx.x; i < nblocks; i += kCosBlock) {
    acc[0] += partial[(int64_t)i * 3 + 0];
    acc[1] += partial[(int64_t)i * 3 + 1];
    acc[2] += partial[(int64_t)i * 3 + 2];
  }
  __shared__ double sh[3][kCosBlock / kWave];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    const double s = wave_sum(acc[t]);
    if (lane == 0) sh[t][wave] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double dot = 0.0, na = 0.0, nb = 0.0;
    for (int w = 0; w < kCosBlock / kWave; ++w) {
      dot += sh[0][w];
      na += sh[1][w];
      nb += sh[2][w];
    }
    double c;
    int dec;
    if (!(isfinite(dot) && isfinite(na) && isfinite(nb))) {
      c = __longlong_as_double(0x7ff8000000000000LL);
      dec = 0;
    } else if (na == 0.0 && nb == 0.0) {
      c = 1.0;
      dec = 1.0 >= gamma ? 1 : 0;
    } else if (na == 0.0 || nb == 0.0) {
      c = 0.0;
      dec = 0.0 >= gamma ? 1 : 0;
    } else {
      const double nrm = __dsqrt_rn(na * nb);
      c = dot / nrm;
      dec = dot >= gamma * nrm ? 1 : 0;
    }
    if (result_cos) *result_cos = c;
    *result_dec = dec;
  }
}

}  // namespace si
