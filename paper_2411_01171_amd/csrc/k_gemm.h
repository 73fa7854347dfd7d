// GEMM kernels of the staged path and their fused epilogues.
//
// Both kernels compute  acc[m, n] = sum_k A[m, k] * Wp[n, k]  where A is the
// token-major activation [M, K] (row stride lda) and Wp the re-laid-out weight
// [N, K] (k contiguous), and hand groups of four consecutive output columns of
// one row to an epilogue functor:  epi(m, n0, v[4])  with n0 % 4 == 0.
//
//   gemm_bf16_kernel  bf16 operands, fp32 accumulation on the matrix cores
//                     (v_mfma_f32_32x32x16_bf16).  The weight tile is the
//                     MFMA's row operand and the activation tile its column
//                     operand, so a lane ends up holding 4 consecutive output
//                     columns of ONE token: bias, GEGLU pairing and vector
//                     stores need no cross-lane traffic.
//   gemm_f32_kernel   fp32 operands on the vector ALUs, for the fp32 block.
#pragma once
#include "si_common.h"
#include "k_norm.h"

namespace si {

// ----------------------------------------------------------------------------- epilogues

// out[m, n] = T(acc + bias[n])
template <typename T>
struct EpiStore {
  static constexpr bool kRows8 = false;
  T* out;
  int64_t ld;
  const T* bias;
  float scale = 1.f;  // applied to acc + bias before the one rounding (the matrix-core attention's query scale)
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    T* p = out + m * ld + n0;
    if constexpr (sizeof(T) == 2) {
      uint2 pk;
      pk.x = (unsigned)float_to_bf16_bits((v[0] + param_or(bias, n0 + 0, 0.f)) * scale) |
             ((unsigned)float_to_bf16_bits((v[1] + param_or(bias, n0 + 1, 0.f)) * scale) << 16);
      pk.y = (unsigned)float_to_bf16_bits((v[2] + param_or(bias, n0 + 2, 0.f)) * scale) |
             ((unsigned)float_to_bf16_bits((v[3] + param_or(bias, n0 + 3, 0.f)) * scale) << 16);
      *reinterpret_cast<uint2*>(p) = pk;
    } else {
      float4 o;
      o.x = (v[0] + param_or(bias, n0 + 0, 0.f)) * scale;
      o.y = (v[1] + param_or(bias, n0 + 1, 0.f)) * scale;
      o.z = (v[2] + param_or(bias, n0 + 2, 0.f)) * scale;
      o.w = (v[3] + param_or(bias, n0 + 3, 0.f)) * scale;
      *reinterpret_cast<float4*>(p) = o;
    }
  }
};

// q/k/v projection for the matrix-core attention kernel: columns [0, 2D) (queries, keys) are stored
// row-major as EpiStore does, the queries multiplied by qscale (softmax scale * log2(e)) in fp32 before
// their one rounding; the value columns go straight to the transposed copy the kernel reads,
// vt[(s*D + c)*Pw + key] for token m = s*Pw + key (keys contiguous), and are not stored row-major.
struct EpiStoreQKVt {
  static constexpr bool kRows8 = false;
  bf16* out;
  int64_t ld;
  bf16* vt;
  int D, Pw;
  float qscale;
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    if (n0 < 2 * D) {
      const float sc = n0 < D ? qscale : 1.f;
      uint2 pk;
      pk.x = (unsigned)float_to_bf16_bits(v[0] * sc) | ((unsigned)float_to_bf16_bits(v[1] * sc) << 16);
      pk.y = (unsigned)float_to_bf16_bits(v[2] * sc) | ((unsigned)float_to_bf16_bits(v[3] * sc) << 16);
      *reinterpret_cast<uint2*>(out + m * ld + n0) = pk;
    } else {
      const int mi = (int)m, s = mi / Pw, key = mi - s * Pw;
      bf16* p = vt + ((int64_t)s * D + (n0 - 2 * D)) * Pw + key;
#pragma unroll
      for (int i = 0; i < 4; ++i) p[(int64_t)i * Pw] = from_float<bf16>(v[i]);
    }
  }
};

// Residual stream (fp32): h[m, n] = (accumulate ? h[m, n] : 0) + acc + bias[n];
// optionally the new value is also stored in copy (operand of proj_out): fp32 storage
// as is; 16-bit storage as fp16 (11 significand bits, saturated at +-65504), row stride ld.
// FRAG: the copy goes to a buffer in the ring kernels' fragment order.
template <typename T, bool FRAG = false>
struct EpiResidual {
  static constexpr bool kRows8 = false;
  float* h;
  int64_t ld;
  const T* bias;
  int accumulate;
  T* copy;
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    float4* p = reinterpret_cast<float4*>(h + m * ld + n0);
    float4 o = accumulate ? *p : make_float4(0.f, 0.f, 0.f, 0.f);
    o.x += v[0] + param_or(bias, n0 + 0, 0.f);
    o.y += v[1] + param_or(bias, n0 + 1, 0.f);
    o.z += v[2] + param_or(bias, n0 + 2, 0.f);
    o.w += v[3] + param_or(bias, n0 + 3, 0.f);
    *p = o;
    if (copy) {
      const float ov[4] = {o.x, o.y, o.z, o.w};
      if constexpr (sizeof(T) == 2) {
        typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
        f16x4_t c4;
#pragma unroll
        for (int i = 0; i < 4; ++i) c4[i] = (_Float16)__builtin_amdgcn_fmed3f(ov[i], -65504.f, 65504.f);
        *reinterpret_cast<f16x4_t*>(copy + (FRAG ? act_offset(m, n0, (int)ld) : m * ld + n0)) = c4;
      } else {
        T* c = copy + m * ld + n0;
#pragma unroll
        for (int i = 0; i < 4; ++i) c[i] = from_float<T>(ov[i]);
      }
    }
  }
};

// GEGLU: the packed weight interleaves value column j (row 2j) with gate column
// j (row 2j+1), so columns (n0, n0+1) and (n0+2, n0+3) are (value, gate) pairs.
// g[m, n0/2 + i] = (value + b1[j]) * gelu_erf(gate + b1[inner + j])
// FRAG: g is a buffer in the ring kernels' fragment order (row width ld).
template <typename T, bool FRAG = false>
struct EpiGeglu {
  static constexpr bool kRows8 = false;
  T* g;
  int64_t ld;
  const T* b1;
  int inner;  // 4D
  // One 32-column result block of the ring kernel at a time (16-bit storage, fragment-order g): the
  // lane holds, per register quad q, the (value, gate) pairs of output channels 4q + 2*half + {0, 1}
  // of the block's 16; one lane^32 exchange per two quads leaves each lane with the 8 consecutive
  // channels of one 16-byte granule (half 0: channels 0..7, half 1: 8..15), so a wavefront's store is
  // one contiguous KiB of the fragment-order buffer instead of four 4-byte pieces per lane.  The
  // GELU is the polynomial of the register-resident kernels.  Called by every lane of the wavefront
  // (the exchange needs them all); rows past the end are not stored.
  static constexpr bool kBlock32 = FRAG && sizeof(T) == 2;
  __device__ __forceinline__ void block32(int64_t m, bool mvalid, int n0, const f32x16_t& acc, int half) const {
    const int j0 = n0 >> 1;  // first of the block's 16 output channels
    unsigned d[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int j = j0 + 4 * q + 2 * half;
      float bv0 = 0.f, bv1 = 0.f, bg0 = 0.f, bg1 = 0.f;
      if (b1) {  // two adjacent 16-bit values per load (j is even, the vector 4-byte aligned)
        const unsigned wv = *reinterpret_cast<const unsigned*>(b1 + j), wg = *reinterpret_cast<const unsigned*>(b1 + inner + j);
        bv0 = __uint_as_float(wv << 16); bv1 = __uint_as_float(wv & 0xffff0000u);
        bg0 = __uint_as_float(wg << 16); bg1 = __uint_as_float(wg & 0xffff0000u);
      }
      const float a0 = (acc[4 * q + 0] + bv0) * gelu_poly(acc[4 * q + 1] + bg0);
      const float a1 = (acc[4 * q + 2] + bv1) * gelu_poly(acc[4 * q + 3] + bg1);
      d[q] = (unsigned)float_to_bf16_bits(a0) | ((unsigned)float_to_bf16_bits(a1) << 16);
    }
    // lanes 32..63 of the first operand change places with lanes 0..31 of the second
    const auto x = __builtin_amdgcn_permlane32_swap(d[0], d[2], false, false);
    const auto y = __builtin_amdgcn_permlane32_swap(d[1], d[3], false, false);
    if (mvalid) {
      u32x4_t o;
      o.x = x[0]; o.y = x[1]; o.z = y[0]; o.w = y[1];
      *reinterpret_cast<u32x4_t*>(reinterpret_cast<unsigned short*>(g) + act_offset(m, j0 + 8 * half, (int)ld)) = o;
    }
  }
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    const int j = n0 >> 1;
    const float a0 = (v[0] + param_or(b1, j, 0.f)) * gelu_erf(v[1] + param_or(b1, inner + j, 0.f));
    const float a1 = (v[2] + param_or(b1, j + 1, 0.f)) * gelu_erf(v[3] + param_or(b1, inner + j + 1, 0.f));
    T* p = g + (FRAG ? act_offset(m, j, (int)ld) : m * ld + j);
    if constexpr (sizeof(T) == 2) {
      *reinterpret_cast<unsigned*>(p) = (unsigned)float_to_bf16_bits(a0) | ((unsigned)float_to_bf16_bits(a1) << 16);
    } else {
      *reinterpret_cast<float2*>(p) = make_float2(a0, a1);
    }
  }
};

// Slice-out: out[b, n, f, p] = x[b, n, f, p] + acc + b_out[n] for token m = (b, f, p)
// of the window; the sum is formed in fp32 and rounded once.
template <typename T>
struct EpiSliceOut {
  static constexpr bool kRows8 = false;
  const T* x;
  T* out;
  const T* bias;
  Window w;
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    const int mi = (int)m;  // window tokens fit 31 bits: 32-bit divisions
    const int pl = mi % w.Pw;
    const int bf = mi / w.Pw;
    const int fl = bf % w.Fw, b = bf / w.Fw;
    const int64_t cs = (int64_t)w.F * w.P;
    const int64_t off = (((int64_t)b * w.C + n0) * w.F + (w.f0 + fl)) * w.P + w.p0 + pl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float r = to_float(x[off + i * cs]) + (v[i] + param_or(bias, n0 + i, 0.f));
      out[off + i * cs] = from_float<T>(r);
    }
  }
};

// ----------------------------------------------------------------------------- bf16 MFMA GEMM

// Block tile BM tokens x BN columns, BK = 64, 256 threads = 4 wavefronts laid out
// WAVES_M x WAVES_N; each wavefront owns (BM/WAVES_M) x (BN/WAVES_N) outputs as
// 32x32 MFMA blocks.  LDS rows are padded by 8 elements (16 bytes) so that the
// 16-byte fragment reads of 32 consecutive rows spread over all banks.  Global
// loads for tile k+1 are issued before the MFMAs of tile k (register staging,
// two LDS buffers, one barrier per tile).  Out-of-range rows / k are zero-filled.
// Requires K % 8 == 0, lda % 8 == 0 and 16-byte aligned bases.
// F16: the 16-bit operands are fp16 (v_mfma_f32_32x32x16_f16) instead of bf16.
template <int BM, int BN, int WAVES_M, int WAVES_N, class Epi, int BK = 64, bool F16 = false>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16* __restrict__ A, int64_t lda,
                                                        const bf16* __restrict__ Wp, int64_t M, int N, int K, Epi epi) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per block");
  constexpr int LDK = BK + 8, CPR = BK / 8;  // 16-byte chunks per tile row
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront tile
  constexpr int TM = WM / 32, TN = WN / 32;            // MFMA blocks per wavefront
  constexpr int A_CHUNKS = BM * CPR / 256, W_CHUNKS = BN * CPR / 256;
  static_assert(WM % 32 == 0 && WN % 32 == 0 && A_CHUNKS >= 1 && W_CHUNKS >= 1, "tile shape");

  __shared__ __attribute__((aligned(16))) unsigned short As[2][BM][LDK];
  __shared__ __attribute__((aligned(16))) unsigned short Ws[2][BN][LDK];

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;

  uint4 ra[A_CHUNKS], rw[W_CHUNKS];
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      const int id = tid + i * 256, row = id / CPR, kc = (id % CPR) * 8;
      const int64_t m = m0 + row;
      ra[i] = (m < M && k0 + kc < K) ? *reinterpret_cast<const uint4*>(A + m * lda + k0 + kc) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
      const int id = tid + i * 256, row = id / CPR, kc = (id % CPR) * 8;
      const int n = n0 + row;
      rw[i] = (n < N && k0 + kc < K) ? *reinterpret_cast<const uint4*>(Wp + (int64_t)n * K + k0 + kc) : make_uint4(0, 0, 0, 0);
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
      *reinterpret_cast<uint4*>(&Ws[buf][row][kc]) = rw[i];
    }
  };

  f32x16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (K + BK - 1) / BK;
  load_tile(0);
  store_tile(0);
  __syncthreads();
  const int frow = lane % 32, fk = (lane / 32) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_tile((kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      u32x4_t wf[TN], af[TM];
#pragma unroll
      for (int i = 0; i < TN; ++i) wf[i] = *reinterpret_cast<const u32x4_t*>(&Ws[cur][wn0 + i * 32 + frow][kk + fk]);
#pragma unroll
      for (int j = 0; j < TM; ++j) af[j] = *reinterpret_cast<const u32x4_t*>(&As[cur][wm0 + j * 32 + frow][kk + fk]);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          if constexpr (F16) {
            typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, wf[i]), __builtin_bit_cast(f16x8_t, af[j]),
                                                               acc[i][j], 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wf[i]), __builtin_bit_cast(bf16x8_t, af[j]),
                                                                acc[i][j], 0, 0, 0);
          }
        }
    }
    if (kt + 1 < nk) store_tile(cur ^ 1);
    __syncthreads();
  }

  // MFMA result layout (32x32): lane holds column (lane % 32) = token, and for
  // register quad q the four consecutive rows 8q + 4*(lane/32) + {0..3} = output columns.
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int64_t m = m0 + wm0 + j * 32 + frow;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn0 + i * 32 + q * 8 + (lane / 32) * 4;
        if (n < N) {
          const float v[4] = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
          epi(m, n, v);
        }
      }
    }
  }
}

// ----------------------------------------------------------------------------- fp32 VALU GEMM

// 64 x 64 block tile, BK = 16, each thread a 4 (tokens) x 4 (columns) micro-tile,
// plain fmaf accumulation in k order.  Any M, N % 4 == 0, any K.
template <class Epi>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t lda, const float* __restrict__ Wp,
                                                       int64_t M, int N, int K, Epi epi) {
  constexpr int BK = 16;
  __shared__ float As[BK][64 + 4];
  __shared__ float Ws[BK][64 + 4];
  const int tid = threadIdx.x;
  const int tn = tid % 16, tm = tid / 16;
  const int64_t m0 = (int64_t)blockIdx.x * 64;
  const int n0 = blockIdx.y * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + i * 256, row = id / BK, k = id % BK;
      const int64_t m = m0 + row;
      const int n = n0 + row;
      As[k][row] = (m < M && k0 + k < K) ? A[m * lda + k0 + k] : 0.f;
      Ws[k][row] = (n < N && k0 + k < K) ? Wp[(int64_t)n * K + k0 + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][tm * 4]);
      const float4 w = *reinterpret_cast<const float4*>(&Ws[k][tn * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
    }
    __syncthreads();
  }
  const int n = n0 + tn * 4;
  if (n >= N) return;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + tm * 4 + i;
    if (m < M) epi(m, n, acc[i]);
  }
}

}  // namespace si
