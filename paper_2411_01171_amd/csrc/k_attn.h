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

}  // namespace si
