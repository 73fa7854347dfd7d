// Normalisation and layout kernels of the staged (general-shape) path:
//   gn_stats_kernel        GroupNorm statistics per (batch, frame, group)     [HBM bound]
//   window_to_tokens_kernel  slice window -> GroupNorm -> token-major rows     [HBM bound]
//   layer_norm_kernel      row LayerNorm (+ frame embedding), fp32 -> T        [HBM/L2 bound]
//   pe_table_kernel        sinusoidal frame embedding table
//   pack_transpose_kernel  [in,out] weight -> [out,in] (k-contiguous) layout
#pragma once
#include "si_common.h"

namespace si {

// Fragment order of a 16-bit activation operand of the ring kernels (k_conv.h): granule
// act_granule(t, c8) holds the 16 bytes (channels 8*c8 .. +7) of token t; a 1 KiB fragment is the
// 64 granules of (32-token block, 16-channel step), 16-channel steps fastest; the buffer starts with
// a 256-byte block of zeros.
constexpr int kActZeroBytes = 256;
__host__ __device__ __forceinline__ int64_t act_granule(int64_t t, int c8, int C) {
  return ((t >> 5) * (C / 16) + (c8 >> 1)) * 64 + (c8 & 1) * 32 + (t & 31);
}
// element offset (16-bit elements) of channel c of token t in such a buffer
__host__ __device__ __forceinline__ int64_t act_offset(int64_t t, int c, int C) {
  return kActZeroBytes / 2 + act_granule(t, c >> 3, C) * 8 + (c & 7);
}

// One block per (b, f, g).  Reduces the n_g * P values x[b, g*n_g:(g+1)*n_g, f, :].
// Sums are taken relative to the group's first element so that a large common
// offset does not cancel in fp32; per-thread fp32 partials are merged in fp64.
// stats[((b*F + f)*G + g)*2 + {0,1}] = {mean, 1/sqrt(var + eps)}.
//
// COS: the same pass also reduces x against a second tensor `key` of the same
// shape (the input of the last recomputed step of the Step Rehash walk):
// partial[block*3 + {0,1,2}] = {<x,key>, |x|^2, |key|^2} over the block's
// elements, exact products and fp64 accumulation as in cosine_partial_kernel,
// so the similarity test costs one extra read of `key` and no extra read of x.
// The GroupNorm sums are the same instructions on the same values either way.
template <typename T, int VEC, bool COS = false>
__global__ __launch_bounds__(256) void gn_stats_kernel(const T* __restrict__ x, float* __restrict__ stats,
                                                       int C, int F, int64_t P, int G, float eps,
                                                       const T* __restrict__ key = nullptr,
                                                       double* __restrict__ partial = nullptr) {
  const int g = blockIdx.x % G;
  const int f = (blockIdx.x / G) % F;
  const int b = blockIdx.x / (G * F);
  const int ng = C / G;
  const int pv = (int)(P / VEC);  // vectors per channel row (VEC divides P; ng*P < 2^31 is checked by the host)
  const T* base = x + (((int64_t)b * C + (int64_t)g * ng) * F + f) * P;
  const int64_t cstride = (int64_t)F * P;
  const float shift = to_float(base[0]);

  float s1 = 0.f, s2 = 0.f;
  double dot = 0.0, na = 0.0, nb = 0.0;
  const T* kbase = COS ? key + (base - x) : nullptr;
  // a thread walks its vectors of every channel row; four rows' loads are in flight at a time.  Short
  // rows (fewer vectors than threads) are shared out so that 256 / vlanes rows are walked side by side.
  int vlanes = 256;
  while (vlanes / 2 >= pv && vlanes > 1) vlanes >>= 1;
  const int v0 = threadIdx.x & (vlanes - 1), c0 = threadIdx.x / vlanes, cstep = 256 / vlanes;
  for (int v = v0; v < pv; v += vlanes)
#pragma unroll 4
  for (int c = c0; c < ng; c += cstep) {
    const T* p = base + c * cstride + (int64_t)v * VEC;
    if constexpr (VEC == 1) {
      const float xv = to_float(p[0]);
      const float d = xv - shift;
      s1 += d;
      s2 += d * d;
      if constexpr (COS) {
        const double da = xv, db = to_float(kbase[c * cstride + v]);
        dot = fma(da, db, dot);
        na = fma(da, da, na);
        nb = fma(db, db, nb);
      }
    } else if constexpr (sizeof(T) == 2) {  // 8 x bf16 = 16 bytes
      const uint4 raw = *reinterpret_cast<const uint4*>(p);
      const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float d0 = __uint_as_float(w[i] << 16) - shift;
        const float d1 = __uint_as_float(w[i] & 0xffff0000u) - shift;
        s1 += d0 + d1;
        s2 += d0 * d0 + d1 * d1;
      }
      if constexpr (COS) {
        const uint4 rk = *reinterpret_cast<const uint4*>(kbase + c * cstride + (int64_t)v * VEC);
        const unsigned wk[4] = {rk.x, rk.y, rk.z, rk.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float a0 = __uint_as_float(w[i] << 16), a1 = __uint_as_float(w[i] & 0xffff0000u);
          const float b0 = __uint_as_float(wk[i] << 16), b1 = __uint_as_float(wk[i] & 0xffff0000u);
          // 8-bit significands: each product is exact in fp32
          dot += (double)(a0 * b0);
          dot += (double)(a1 * b1);
          na += (double)(a0 * a0);
          na += (double)(a1 * a1);
          nb += (double)(b0 * b0);
          nb += (double)(b1 * b1);
        }
      }
    } else {  // 4 x f32 = 16 bytes
      const float4 raw = *reinterpret_cast<const float4*>(p);
      const float d0 = raw.x - shift, d1 = raw.y - shift, d2 = raw.z - shift, d3 = raw.w - shift;
      s1 += (d0 + d1) + (d2 + d3);
      s2 += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
      if constexpr (COS) {
        const float4 rk = *reinterpret_cast<const float4*>(kbase + c * cstride + (int64_t)v * VEC);
        const float fa[4] = {raw.x, raw.y, raw.z, raw.w}, fb[4] = {rk.x, rk.y, rk.z, rk.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const double da = fa[i], db = fb[i];
          dot = fma(da, db, dot);
          na = fma(da, da, na);
          nb = fma(db, db, nb);
        }
      }
    }
  }
  if constexpr (COS) {
    dot = wave_sum(dot);
    na = wave_sum(na);
    nb = wave_sum(nb);
    __shared__ double shc[3][4];
    if (threadIdx.x % kWave == 0) {
      shc[0][threadIdx.x / kWave] = dot;
      shc[1][threadIdx.x / kWave] = na;
      shc[2][threadIdx.x / kWave] = nb;
    }
    __syncthreads();
    if (threadIdx.x < 3)
      partial[(int64_t)blockIdx.x * 3 + threadIdx.x] =
          (shc[threadIdx.x][0] + shc[threadIdx.x][1]) + (shc[threadIdx.x][2] + shc[threadIdx.x][3]);
  }
  double a1 = wave_sum((double)s1), a2 = wave_sum((double)s2);
  __shared__ double sh[2][4];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (lane == 0) {
    sh[0][wave] = a1;
    sh[1][wave] = a2;
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

// Geometry of one slice window and of the token order used inside a slice:
// token m = (b*Fw + (f - f0))*Pw + (p - p0).
struct Window {
  int B, C, F;   // full tensor
  int64_t P;     // H*W
  int f0, Fw;    // frame window
  int64_t p0;    // first position
  int Pw;        // positions in the window
  int G;         // GroupNorm groups
};

// Slice-in: a0[m, c] = GN(x)[b, c, f, p] for the window's tokens.  64 x 64
// (position x channel) tiles are transposed through LDS so that both the read
// (along positions) and the write (along channels) are contiguous.  Used for fp32
// storage; 16-bit storage takes window_to_tokens_f16_kernel.
template <typename T>
__global__ __launch_bounds__(256) void window_to_tokens_kernel(const T* __restrict__ x, const float* __restrict__ stats,
                                                               const T* __restrict__ gamma, const T* __restrict__ beta,
                                                               T* __restrict__ a0, Window w) {
  __shared__ float tile[64][65];
  const int bf = blockIdx.z;  // b*Fw + fl
  const int b = bf / w.Fw, fl = bf % w.Fw, f = w.f0 + fl;
  const int pt = blockIdx.x * 64, ct = blockIdx.y * 64;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  const int ng = w.C / w.G;
#pragma unroll 4
  for (int cl = ty; cl < 64; cl += 4) {
    const int c = ct + cl, pl = pt + tx;
    float v = 0.f;
    if (c < w.C && pl < w.Pw) {
      const int g = c / ng;
      const float mean = stats[(((int64_t)b * w.F + f) * w.G + g) * 2 + 0];
      const float rstd = stats[(((int64_t)b * w.F + f) * w.G + g) * 2 + 1];
      const float xv = to_float(x[(((int64_t)b * w.C + c) * w.F + f) * w.P + w.p0 + pl]);
      v = (xv - mean) * rstd * param_or(gamma, c, 1.f) + param_or(beta, c, 0.f);
    }
    tile[cl][tx] = v;
  }
  __syncthreads();
#pragma unroll 4
  for (int pl = ty; pl < 64; pl += 4) {
    const int c = ct + tx, p = pt + pl;
    if (c < w.C && p < w.Pw) {
      const int64_t m = (int64_t)bf * w.Pw + p;
      a0[m * w.C + c] = from_float<T>(tile[tx][pl]);
    }
  }
}

// Slice-in for bf16 storage: the normalised value (bounded by construction) is kept as fp16, the
// operand type of proj_in on this path -- three more significand bits than bf16 for the same bytes.
// 8-byte reads along positions (when the frame size and the window start are multiples of 4
// positions), 16-byte writes of 8 channels.  C % 8 == 0; row m holds C values, or (FRAG) the
// buffer is in the ring kernels' fragment order.
template <bool FRAG>
__global__ __launch_bounds__(256) void window_to_tokens_f16_kernel(const bf16* __restrict__ x, const float* __restrict__ stats,
                                                                     const bf16* __restrict__ gamma, const bf16* __restrict__ beta,
                                                                     bf16* __restrict__ a0, Window w) {
  __shared__ float tile[64][65];
  const int bf = blockIdx.z;
  const int b = bf / w.Fw, fl = bf % w.Fw, f = w.f0 + fl;
  const int pt = blockIdx.x * 64, ct = blockIdx.y * 64;
  const int ng = w.C / w.G;
  const bool vec_ok = (w.P % 4 == 0) && (w.p0 % 4 == 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int id = threadIdx.x + i * 256, cl = id / 16, pq = (id % 16) * 4;
    const int c = ct + cl, pl = pt + pq;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (c < w.C && pl < w.Pw) {
      const int g = c / ng;
      const float mean = stats[(((int64_t)b * w.F + f) * w.G + g) * 2 + 0];
      const float rstd = stats[(((int64_t)b * w.F + f) * w.G + g) * 2 + 1];
      const float ga = param_or(gamma, c, 1.f), be = param_or(beta, c, 0.f);
      const bf16* src = x + (((int64_t)b * w.C + c) * w.F + f) * w.P + w.p0 + pl;
      float xv[4] = {0.f, 0.f, 0.f, 0.f};
      if (vec_ok && pl + 3 < w.Pw) {
        const uint2 raw = *reinterpret_cast<const uint2*>(src);
        xv[0] = __uint_as_float(raw.x << 16);
        xv[1] = __uint_as_float(raw.x & 0xffff0000u);
        xv[2] = __uint_as_float(raw.y << 16);
        xv[3] = __uint_as_float(raw.y & 0xffff0000u);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (pl + j < w.Pw) xv[j] = to_float(src[j]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = (xv[j] - mean) * rstd * ga + be;  // same expression as window_to_tokens_kernel
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) tile[cl][pq + j] = v[j];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int id = threadIdx.x + i * 256, pl = id / 8, co = (id % 8) * 8;
    const int p = pt + pl, c = ct + co;
    if (p < w.Pw && c < w.C) {
      typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
      f16x8_t o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = (_Float16)__builtin_amdgcn_fmed3f(tile[co + j][pl], -65504.f, 65504.f);
      const int64_t m = (int64_t)bf * w.Pw + p;
      *reinterpret_cast<f16x8_t*>(a0 + (FRAG ? act_offset(m, c, w.C) : m * w.C + c)) = o;
    }
  }
}

// PE[f, 2i] = sin(f / 10000^(2i/D)), PE[f, 2i+1] = cos(same), evaluated in fp64.
__global__ void pe_table_kernel(float* __restrict__ pe, int F, int D) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= F * D) return;
  const int f = idx / D, i = idx % D;
  const int even = i - (i & 1);
  const double angle = (double)f / pow(10000.0, (double)even / (double)D);
  pe[idx] = (float)((i & 1) ? cos(angle) : sin(angle));
}

// Row LayerNorm of the fp32 residual stream; one wavefront per row, the row is
// held in registers (D <= 2048, D % 4 == 0).  Optional frame embedding: row m
// belongs to frame f0 + (m / Pw) % Fw.
// FRAG (16-bit T): the output is written in the ring kernels' fragment order instead of rows of D.
template <typename T, bool FRAG = false>
__global__ __launch_bounds__(256) void layer_norm_kernel(const float* __restrict__ h, T* __restrict__ a, int64_t M, int D,
                                                         const T* __restrict__ gamma, const T* __restrict__ beta, float eps,
                                                         const float* __restrict__ pe, int Pw, int Fw, int f0) {
  const int lane = threadIdx.x % kWave;
  const int64_t m = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (m >= M) return;
  const float4* row = reinterpret_cast<const float4*>(h + m * D);
  const int nv = D / 4;
  float4 r[8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int v = lane + i * kWave;
    if (v < nv) {
      r[i] = row[v];
      s += (r[i].x + r[i].y) + (r[i].z + r[i].w);
    }
  }
  const float mean = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int v = lane + i * kWave;
    if (v < nv) {
      const float dx = r[i].x - mean, dy = r[i].y - mean, dz = r[i].z - mean, dw = r[i].w - mean;
      q += (dx * dx + dy * dy) + (dz * dz + dw * dw);
    }
  }
  const float rstd = rsqrtf(wave_sum(q) / (float)D + eps);
  const float* perow = nullptr;
  if (pe) perow = pe + (int64_t)(f0 + (int)((m / Pw) % Fw)) * D;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int v = lane + i * kWave;
    if (v < nv) {
      const float in[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
      float y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = v * 4 + e;
        y[e] = (in[e] - mean) * rstd * param_or(gamma, c, 1.f) + param_or(beta, c, 0.f);
        if (perow) y[e] += perow[c];
      }
      // four consecutive channels per store (rows start 8- / 16-byte aligned: D % 4 == 0)
      if constexpr (sizeof(T) == 2) {
        uint2 pk;
        pk.x = (unsigned)float_to_bf16_bits(y[0]) | ((unsigned)float_to_bf16_bits(y[1]) << 16);
        pk.y = (unsigned)float_to_bf16_bits(y[2]) | ((unsigned)float_to_bf16_bits(y[3]) << 16);
        *reinterpret_cast<uint2*>(a + (FRAG ? act_offset(m, v * 4, D) : m * D + v * 4)) = pk;
      } else {
        *reinterpret_cast<float4*>(a + m * D + v * 4) = make_float4(y[0], y[1], y[2], y[3]);
      }
    }
  }
}

// Row LayerNorm into the ring kernels' fragment order for windows of few rows (bf16, D % 8 == 0,
// D <= 2048): one wavefront per row as in layer_norm_kernel (as many wavefronts as rows), eight
// consecutive rows per workgroup.  The eight normalised rows meet in LDS, and the workgroup writes
// them as whole 128-byte pieces of the fragment-order buffer (8 tokens x the 16 bytes of one
// 8-channel granule) instead of 16-byte pieces per row; gain and shift are read four at a time.
// Same arithmetic per element as layer_norm_kernel.
__global__ __launch_bounds__(512) void layer_norm_rows8_kernel(const float* __restrict__ h, bf16* __restrict__ a, int64_t M, int D,
                                                               const bf16* __restrict__ gamma, const bf16* __restrict__ beta, float eps,
                                                               const float* __restrict__ pe, int Pw, int Fw, int f0) {
  constexpr int LDR = 2048 + 8;  // 16-bit elements per LDS row: 16-byte aligned rows that rotate over the banks
  __shared__ __attribute__((aligned(16))) unsigned short tile[8][LDR];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t m0 = (int64_t)blockIdx.x * 8, m = m0 + wave;
  if (m < M) {
    const float4* row = reinterpret_cast<const float4*>(h + m * D);
    const int nv = D / 4;
    float4 r[8];
    uint2 gr[8], br[8];  // gain and shift are requested together with the row: their latency hides behind the two sums
    const float* perow = pe ? pe + (int64_t)(f0 + (int)((m / Pw) % Fw)) * D : nullptr;
    float4 pr[8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = lane + i * kWave;
      if (v < nv) {
        r[i] = row[v];
        gr[i] = gamma ? *reinterpret_cast<const uint2*>(gamma + v * 4) : make_uint2(0x3f803f80u, 0x3f803f80u);
        br[i] = beta ? *reinterpret_cast<const uint2*>(beta + v * 4) : make_uint2(0u, 0u);
        pr[i] = perow ? *reinterpret_cast<const float4*>(perow + v * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = lane + i * kWave;
      if (v < nv) s += (r[i].x + r[i].y) + (r[i].z + r[i].w);
    }
    const float mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = lane + i * kWave;
      if (v < nv) {
        const float dx = r[i].x - mean, dy = r[i].y - mean, dz = r[i].z - mean, dw = r[i].w - mean;
        q += (dx * dx + dy * dy) + (dz * dz + dw * dw);
      }
    }
    const float rstd = rsqrtf(wave_sum(q) / (float)D + eps);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = lane + i * kWave;
      if (v < nv) {
        const float in[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
        const float g[4] = {__uint_as_float(gr[i].x << 16), __uint_as_float(gr[i].x & 0xffff0000u), __uint_as_float(gr[i].y << 16),
                            __uint_as_float(gr[i].y & 0xffff0000u)};
        const float b[4] = {__uint_as_float(br[i].x << 16), __uint_as_float(br[i].x & 0xffff0000u), __uint_as_float(br[i].y << 16),
                            __uint_as_float(br[i].y & 0xffff0000u)};
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (in[e] - mean) * rstd * g[e] + b[e];
        if (perow) {
          y[0] += pr[i].x; y[1] += pr[i].y; y[2] += pr[i].z; y[3] += pr[i].w;
        }
        uint2 pk;
        pk.x = (unsigned)float_to_bf16_bits(y[0]) | ((unsigned)float_to_bf16_bits(y[1]) << 16);
        pk.y = (unsigned)float_to_bf16_bits(y[2]) | ((unsigned)float_to_bf16_bits(y[3]) << 16);
        *reinterpret_cast<uint2*>(&tile[wave][v * 4]) = pk;
      }
    }
  }
  __syncthreads();
  const int items = (D / 8) * 8;  // (8-channel granule, row) pairs; the 8 rows of a granule are 128 contiguous bytes
  for (int idx = threadIdx.x; idx < items; idx += 512) {
    const int c8 = idx / 8, t = idx % 8;
    if (m0 + t < M)
      *reinterpret_cast<uint4*>(a + act_offset(m0 + t, c8 * 8, D)) = *reinterpret_cast<const uint4*>(&tile[t][c8 * 8]);
  }
}

// Row LayerNorm into the ring kernels' fragment order (bf16 blocks with D % 32 == 0): one wavefront
// per 8 consecutive rows.  Lane (r = lane % 8, q = lane / 8) owns the channel quads q, q + 8, ... of
// row r, so a load instruction covers 128 contiguous bytes of each of the 8 rows (all of them in
// flight before the first use) and a store instruction writes four complete 128-byte pieces of the
// fragment-order buffer (8 tokens x 16 bytes each).  Row sums meet over the 8 lanes of a row
// (lane ^ 8, 16, 32).  NQ = D / 32 quads per lane.  Same arithmetic per element as layer_norm_kernel.
template <int NQ>
__global__ __launch_bounds__(64) void layer_norm_frag_kernel(const float* __restrict__ h, bf16* __restrict__ a, int64_t M,
                                                             const bf16* __restrict__ gamma, const bf16* __restrict__ beta, float eps,
                                                             const float* __restrict__ pe, int Pw, int Fw, int f0) {
  constexpr int D = 32 * NQ;
  const int lane = threadIdx.x, r = lane % 8, q = lane / 8;
  const int64_t m = (int64_t)blockIdx.x * 8 + r;
  const int64_t ml = m < M ? m : M - 1;  // rows past the end repeat the last one and are not stored
  const float4* row = reinterpret_cast<const float4*>(h + ml * D) + q;
  float4 v[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) v[i] = row[8 * i];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NQ; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  s += __shfl_xor(s, 8, kWave);
  s += __shfl_xor(s, 16, kWave);
  s += __shfl_xor(s, 32, kWave);
  const float mean = s / (float)D;
  float qs = 0.f;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const float dx = v[i].x - mean, dy = v[i].y - mean, dz = v[i].z - mean, dw = v[i].w - mean;
    qs += (dx * dx + dy * dy) + (dz * dz + dw * dw);
  }
  qs += __shfl_xor(qs, 8, kWave);
  qs += __shfl_xor(qs, 16, kWave);
  qs += __shfl_xor(qs, 32, kWave);
  const float rstd = rsqrtf(qs / (float)D + eps);
  const float* perow = pe ? pe + (int64_t)(f0 + (int)((ml / Pw) % Fw)) * D : nullptr;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int c = 4 * (q + 8 * i);
    const float in[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    float ga[4] = {1.f, 1.f, 1.f, 1.f}, be[4] = {0.f, 0.f, 0.f, 0.f}, pv[4] = {0.f, 0.f, 0.f, 0.f};
    if (gamma) {  // four consecutive 16-bit values: one 8-byte load (c % 4 == 0, 16-byte aligned base)
      const uint2 w2 = *reinterpret_cast<const uint2*>(gamma + c);
      ga[0] = __uint_as_float(w2.x << 16); ga[1] = __uint_as_float(w2.x & 0xffff0000u);
      ga[2] = __uint_as_float(w2.y << 16); ga[3] = __uint_as_float(w2.y & 0xffff0000u);
    }
    if (beta) {
      const uint2 w2 = *reinterpret_cast<const uint2*>(beta + c);
      be[0] = __uint_as_float(w2.x << 16); be[1] = __uint_as_float(w2.x & 0xffff0000u);
      be[2] = __uint_as_float(w2.y << 16); be[3] = __uint_as_float(w2.y & 0xffff0000u);
    }
    if (perow) {
      const float4 p4 = *reinterpret_cast<const float4*>(perow + c);
      pv[0] = p4.x; pv[1] = p4.y; pv[2] = p4.z; pv[3] = p4.w;
    }
    float y[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      y[e] = (in[e] - mean) * rstd * ga[e] + be[e];
      if (perow) y[e] += pv[e];
    }
    uint2 pk;
    pk.x = (unsigned)float_to_bf16_bits(y[0]) | ((unsigned)float_to_bf16_bits(y[1]) << 16);
    pk.y = (unsigned)float_to_bf16_bits(y[2]) | ((unsigned)float_to_bf16_bits(y[3]) << 16);
    if (m < M) *reinterpret_cast<uint2*>(a + act_offset(m, c, D)) = pk;
  }
}

// dst[r * ld_dst + k] = src[k * ld_src + col(r)] for r in [0, rows): the k-contiguous
// layout the GEMM kernels read (ld_dst > K lets two copies sit side by side for
// operands that arrive as high/low pairs).  col(r) = col0 + r, or, with `interleave` > 0
// (GEGLU projection), even r -> value column r/2, odd r -> gate column interleave + r/2.
// to_f16 (16-bit T only): the bf16 values are stored as fp16 (weights of the GEMMs whose activation
// operand is fp16; exact for normal fp16 magnitudes, saturated at +-65504).
// frag_tn > 0: the destination is the ring kernels' weight fragment stream for column tiles of
// frag_tn*32 rows of the whole [N, frag_K] matrix; this call fills rows frag_row0 .. of it: element
// (n, k) sits at weight_fragment_index(n, k, frag_K, frag_tn).
__host__ __device__ __forceinline__ int64_t weight_fragment_index(int n, int k, int K, int TN) {
  const int col = n / (32 * TN), i = (n / 32) % TN, lrow = n % 32;
  const int kt = k / 32, ks = (k % 32) / 16, half = (k % 16) / 8, e = k % 8;
  return ((((int64_t)col * (K / 32) + kt) * 2 + ks) * TN + i) * 512 + (half * 32 + lrow) * 8 + e;
}

template <typename T>
__global__ __launch_bounds__(256) void pack_transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int K, int ld_src,
                                                             int rows, int col0, int interleave, int ld_dst, int to_f16 = 0,
                                                             int frag_tn = 0, int frag_row0 = 0, int frag_K = 0) {
  __shared__ T tile[32][33];
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8
  const int r0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
  for (int kk = ty; kk < 32; kk += 8) {
    const int r = r0 + tx, k = k0 + kk;
    if (r < rows && k < K) {
      const int col = interleave > 0 ? ((r & 1) ? interleave + (r >> 1) : (r >> 1)) : col0 + r;
      tile[kk][tx] = src[(int64_t)k * ld_src + col];
    }
  }
  __syncthreads();
  for (int rr = ty; rr < 32; rr += 8) {
    const int r = r0 + rr, k = k0 + tx;
    if (r < rows && k < K) {
      T v = tile[tx][rr];
      if constexpr (sizeof(T) == 2) {
        if (to_f16) v.v = __builtin_bit_cast(unsigned short, (_Float16)__builtin_amdgcn_fmed3f(to_float(v), -65504.f, 65504.f));
      }
      if (frag_tn > 0) dst[weight_fragment_index(frag_row0 + r, k, frag_K, frag_tn)] = v;
      else dst[(int64_t)r * ld_dst + k] = v;
    }
  }
}

// pack_transpose_kernel for 16-bit elements with 64 x 64 tiles: every thread has 8 reads in flight
// (4 bytes where two destination rows are neighbours in the source) and writes whole 16-byte
// granules (8 consecutive k of one row) -- 128 bytes per row per tile in the k-contiguous layout,
// 512 contiguous bytes per 32 rows in a fragment stream.  Requires K % 8 == 0, ld_dst % 8 == 0 and a
// 16-byte aligned destination; same arguments otherwise (col0 = 0).
// One matrix of a batch: the arguments of pack_transpose16_kernel plus the matrix's range of blocks.
struct PackJob {
  const unsigned short* src;
  unsigned short* dst;
  int K, ld_src, rows, interleave, ld_dst, to_f16, frag_tn, frag_row0, frag_K;
  int block0, blocks_x;  // first block of the matrix in the batch's grid; blocks along its rows
};
constexpr int kPackBatchMax = 16;
struct PackBatch {
  PackJob job[kPackBatchMax];
  int n, blocks;
};

__device__ __forceinline__ void pack_transpose16_tile(unsigned short (*tile)[66], const unsigned short* __restrict__ src,
                                                      unsigned short* __restrict__ dst, int K, int ld_src, int rows, int interleave,
                                                      int ld_dst, int to_f16, int frag_tn, int frag_row0, int frag_K, int bx, int by) {
  const int tid = threadIdx.x;
  const int r0 = bx * 64, k0 = by * 64;
  const int rp = 2 * (tid % 32);  // the thread's pair of destination rows within the tile
  const bool pair = interleave == 0 && (ld_src & 1) == 0 && (reinterpret_cast<uintptr_t>(src) & 3) == 0 && r0 + rp + 1 < rows;
  unsigned v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = k0 + tid / 32 + 8 * i, r = r0 + rp;
    v[i] = 0u;
    if (k < K) {
      const unsigned short* row = src + (int64_t)k * ld_src;
      if (pair) {
        v[i] = *reinterpret_cast<const unsigned*>(row + r);
      } else {
        if (r < rows) v[i] = row[interleave > 0 ? (r >> 1) : r];
        if (r + 1 < rows) v[i] |= (unsigned)row[interleave > 0 ? interleave + (r >> 1) : r + 1] << 16;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<unsigned*>(&tile[tid / 32 + 8 * i][rp]) = v[i];
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int g = tid + 256 * j;
    // fragment stream: consecutive lanes take consecutive rows (consecutive granules of a fragment);
    // k-contiguous rows: consecutive lanes take consecutive granules of one row
    const int rl = frag_tn > 0 ? g % 64 : g / 8, k8 = frag_tn > 0 ? g / 64 : g % 8;
    const int r = r0 + rl, k = k0 + 8 * k8;
    if (r >= rows || k >= K) continue;
    unsigned short e[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      e[q] = tile[8 * k8 + q][rl];
      if (to_f16)
        e[q] = __builtin_bit_cast(unsigned short, (_Float16)__builtin_amdgcn_fmed3f(__uint_as_float((unsigned)e[q] << 16), -65504.f, 65504.f));
    }
    uint4 o;
    o.x = e[0] | ((unsigned)e[1] << 16);
    o.y = e[2] | ((unsigned)e[3] << 16);
    o.z = e[4] | ((unsigned)e[5] << 16);
    o.w = e[6] | ((unsigned)e[7] << 16);
    const int64_t at = frag_tn > 0 ? weight_fragment_index(frag_row0 + r, k, frag_K, frag_tn) : (int64_t)r * ld_dst + k;
    *reinterpret_cast<uint4*>(dst + at) = o;
  }
}

__global__ __launch_bounds__(256) void pack_transpose16_kernel(const unsigned short* __restrict__ src,
                                                               unsigned short* __restrict__ dst, int K, int ld_src, int rows,
                                                               int interleave, int ld_dst, int to_f16, int frag_tn,
                                                               int frag_row0, int frag_K) {
  __shared__ unsigned short tile[64][66];  // [k][r]
  pack_transpose16_tile(tile, src, dst, K, ld_src, rows, interleave, ld_dst, to_f16, frag_tn, frag_row0, frag_K, blockIdx.x, blockIdx.y);
}

// All the matrices of a block's weight re-layout in one launch: block b works on the matrix whose
// block range holds b.
__global__ __launch_bounds__(256) void pack_transpose16_batch_kernel(PackBatch b) {
  __shared__ unsigned short tile[64][66];
  int j = 0;
  while (j + 1 < b.n && (int)blockIdx.x >= b.job[j + 1].block0) ++j;
  const PackJob& q = b.job[j];
  const int local = (int)blockIdx.x - q.block0;
  pack_transpose16_tile(tile, q.src, q.dst, q.K, q.ld_src, q.rows, q.interleave, q.ld_dst, q.to_f16, q.frag_tn, q.frag_row0, q.frag_K,
                        local % q.blocks_x, local / q.blocks_x);
}

}  // namespace si
