// Attention kernels.
//
// Sequences are described by strides so that one kernel serves the three uses:
//   temporal self-attention  sequence (b, p): rows b*Fw*Pw + p + i*Pw, i < F
//   spatial self-attention   sequence (b, f): rows (b*Fw + f)*Pw + i,  i < P
//   cross-attention          queries as spatial; keys/values = context rows of b
// Row r of sequence s:  base(s) + i*row_stride,  base(s) = (s / inner)*outer_stride
// + (s % inner)*inner_stride, separately for the query side and the key side.
#pragma once
#include "si_common.h"

namespace si {

struct SeqMap {
  int inner;
  int64_t outer_stride, inner_stride, row_stride;
  __device__ __forceinline__ int64_t row(int s, int i) const {
    return (int64_t)(s / inner) * outer_stride + (int64_t)(s % inner) * inner_stride + (int64_t)i * row_stride;
  }
};

struct AttnArgs {
  const void *q, *k, *v;  // element type T; head h occupies columns [h*d, (h+1)*d)
  void* o;
  int64_t ldq, ldk, ldv, ldo;
  SeqMap qmap, kmap;
  int S, heads, d, Nq, Nk;
  float scale;
};

// Plain vector-ALU attention with an online (running max / running sum) softmax.
// One wavefront serves QB queries of one (sequence, head): in the score phase
// each lane owns one key of a 64-key chunk and forms QB dot products; in the
// value phase each lane owns channels lane and lane+64 (d <= 128).  Exact expf,
// fp32 throughout: this is the path of the fp32 block and the fallback for
// shapes the matrix-core kernels do not cover.
template <typename T, int QB>
__global__ __launch_bounds__(256) void attn_valu_kernel(AttnArgs a) {
  __shared__ float qs[4][QB][128];
  __shared__ float ps[4][QB][kWave];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int s = blockIdx.z, head = blockIdx.y;
  const int q0 = (blockIdx.x * 4 + wave) * QB;
  if (q0 >= a.Nq) return;  // whole wavefront leaves; no block-wide barrier is used below
  const T* Q = static_cast<const T*>(a.q);
  const T* Kp = static_cast<const T*>(a.k);
  const T* Vp = static_cast<const T*>(a.v);
  T* O = static_cast<T*>(a.o);
  const int d = a.d, hc = head * d;

  for (int i = lane; i < QB * d; i += kWave) {
    const int qi = i / d, c = i % d;
    float v = 0.f;
    if (q0 + qi < a.Nq) v = to_float(Q[a.qmap.row(s, q0 + qi) * a.ldq + hc + c]) * a.scale;
    qs[wave][qi][c] = v;
  }
  __builtin_amdgcn_wave_barrier();  // LDS operations of one wavefront complete in program order

  float mrun[QB], lrun[QB], o0[QB], o1[QB];
#pragma unroll
  for (int qi = 0; qi < QB; ++qi) {
    mrun[qi] = -INFINITY;
    lrun[qi] = 0.f;
    o0[qi] = 0.f;
    o1[qi] = 0.f;
  }
  const int c0 = lane, c1 = lane + kWave;
  for (int kc = 0; kc < a.Nk; kc += kWave) {
    const int kj = kc + lane;
    const bool valid = kj < a.Nk;
    float sc[QB];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) sc[qi] = 0.f;
    if (valid) {
      const T* krow = Kp + a.kmap.row(s, kj) * a.ldk + hc;
      for (int c = 0; c < d; ++c) {
        const float kv = to_float(krow[c]);
#pragma unroll
        for (int qi = 0; qi < QB; ++qi) sc[qi] = fmaf(qs[wave][qi][c], kv, sc[qi]);
      }
    }
    float alpha[QB];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
      const float cm = wave_max(valid ? sc[qi] : -INFINITY);
      const float mn = fmaxf(mrun[qi], cm);
      const float p = valid ? expf(sc[qi] - mn) : 0.f;
      alpha[qi] = expf(mrun[qi] - mn);  // first chunk: exp(-inf) = 0
      lrun[qi] = lrun[qi] * alpha[qi] + wave_sum(p);
      mrun[qi] = mn;
      ps[wave][qi][lane] = p;
      o0[qi] *= alpha[qi];
      o1[qi] *= alpha[qi];
    }
    __builtin_amdgcn_wave_barrier();
    const int nvalid = min(kWave, a.Nk - kc);
    for (int j = 0; j < nvalid; ++j) {
      const T* vrow = Vp + a.kmap.row(s, kc + j) * a.ldv + hc;
      const float v0 = c0 < d ? to_float(vrow[c0]) : 0.f;
      const float v1 = c1 < d ? to_float(vrow[c1]) : 0.f;
#pragma unroll
      for (int qi = 0; qi < QB; ++qi) {
        const float p = ps[wave][qi][j];
        o0[qi] = fmaf(p, v0, o0[qi]);
        o1[qi] = fmaf(p, v1, o1[qi]);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
#pragma unroll
  for (int qi = 0; qi < QB; ++qi) {
    if (q0 + qi >= a.Nq) continue;
    T* orow = O + a.qmap.row(s, q0 + qi) * a.ldo + hc;
    const float inv = 1.f / lrun[qi];
    if (c0 < d) orow[c0] = from_float<T>(o0[qi] * inv);
    if (c1 < d) orow[c1] = from_float<T>(o1[qi] * inv);
  }
}

// Short sequences in 16-bit storage (temporal blocks on the staged path: at most 32 tokens per
// sequence, head dimension DH): one wavefront per (sequence, head).  The head's key and value rows
// are staged in LDS; lane l owns query l % 32 and, by its half l / 32, every other key in the score
// phase (the two halves meet in one lane^32 exchange for the row maximum and the row sum) and one
// half of the head's channels in the value phase (the other half's probabilities arrive by the same
// exchange).  fp32 arithmetic, exact expf, as in attn_valu_kernel.
template <int DH>
__global__ __launch_bounds__(256) void attn_short_kernel(AttnArgs a) {
  static_assert(DH % 16 == 0 && DH <= 128, "head dimension");
  constexpr int LD = DH + 8;  // 16-bit elements per LDS row: rows stay 16-byte aligned and rotate over the banks
  __shared__ __attribute__((aligned(16))) unsigned short kv[4][2][32][LD];
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int pair = blockIdx.x * 4 + wave;  // heads fastest: the wavefronts of a workgroup share token rows
  if (pair >= a.S * a.heads) return;       // whole wavefront leaves; no block-wide barrier below
  const int s = pair / a.heads, hc = (pair % a.heads) * DH;
  const int F = a.Nk;
  const unsigned short* Q = static_cast<const unsigned short*>(a.q);
  const unsigned short* Kp = static_cast<const unsigned short*>(a.k);
  const unsigned short* Vp = static_cast<const unsigned short*>(a.v);
  unsigned short* O = static_cast<unsigned short*>(a.o);

  constexpr int LPR = DH / 8, RPI = kWave / LPR;  // lanes per row, rows per wavefront load
  for (int r0 = 0; r0 < F; r0 += RPI) {
    const int r = r0 + lane / LPR, c = (lane % LPR) * 8;
    if (lane < RPI * LPR && r < F) {
      const int64_t row = a.kmap.row(s, r);
      *reinterpret_cast<uint4*>(&kv[wave][0][r][c]) = *reinterpret_cast<const uint4*>(Kp + row * a.ldk + hc + c);
      *reinterpret_cast<uint4*>(&kv[wave][1][r][c]) = *reinterpret_cast<const uint4*>(Vp + row * a.ldv + hc + c);
    }
  }
  const int i = lane % 32, half = lane / 32;
  const bool active = i < a.Nq;
  float q[DH];
  {
    const unsigned short* qrow = Q + a.qmap.row(s, active ? i : 0) * a.ldq + hc;
#pragma unroll
    for (int c = 0; c < DH; c += 8) {
      const uint4 raw = *reinterpret_cast<const uint4*>(qrow + c);
      const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        q[c + 2 * e] = __uint_as_float(w[e] << 16) * a.scale;
        q[c + 2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u) * a.scale;
      }
    }
  }
  __builtin_amdgcn_wave_barrier();  // LDS operations of one wavefront complete in program order

  float sc[16];
  float m = -INFINITY;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    sc[t] = -INFINITY;
    if (2 * t < F) {  // uniform
      const int j = 2 * t + half;
      if (j < F) {
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < DH; c += 8) {
          const uint4 raw = *reinterpret_cast<const uint4*>(&kv[wave][0][j][c]);
          const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc = fmaf(q[c + 2 * e], __uint_as_float(w[e] << 16), acc);
            acc = fmaf(q[c + 2 * e + 1], __uint_as_float(w[e] & 0xffff0000u), acc);
          }
        }
        sc[t] = acc;
      }
      m = fmaxf(m, sc[t]);
    }
  }
  m = fmaxf(m, __shfl_xor(m, 32, kWave));
  float l = 0.f;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    sc[t] = 2 * t < F ? expf(sc[t] - m) : 0.f;  // a key beyond the sequence: exp(-inf) = 0
    l += sc[t];
  }
  l += __shfl_xor(l, 32, kWave);

  constexpr int HC = DH / 2;  // channels of this lane in the value phase: half * HC .. + HC
  float o[HC];
#pragma unroll
  for (int c = 0; c < HC; ++c) o[c] = 0.f;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    if (2 * t < F) {  // uniform
      const float other = __shfl_xor(sc[t], 32, kWave);
      const float pj[2] = {half ? other : sc[t], half ? sc[t] : other};  // keys 2t and 2t + 1
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (2 * t + u < F) {  // uniform
#pragma unroll
          for (int c = 0; c < HC; c += 8) {
            const uint4 raw = *reinterpret_cast<const uint4*>(&kv[wave][1][2 * t + u][half * HC + c]);
            const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              o[c + 2 * e] = fmaf(pj[u], __uint_as_float(w[e] << 16), o[c + 2 * e]);
              o[c + 2 * e + 1] = fmaf(pj[u], __uint_as_float(w[e] & 0xffff0000u), o[c + 2 * e + 1]);
            }
          }
        }
      }
    }
  }
  if (!active) return;
  const float inv = 1.f / l;
  unsigned short* orow = O + a.qmap.row(s, i) * a.ldo + hc + half * HC;
#pragma unroll
  for (int c = 0; c < HC; c += 8) {
    unsigned w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      w[e] = (unsigned)float_to_bf16_bits(o[c + 2 * e] * inv) | ((unsigned)float_to_bf16_bits(o[c + 2 * e + 1] * inv) << 16);
    *reinterpret_cast<uint4*>(orow + c) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

}  // namespace si
