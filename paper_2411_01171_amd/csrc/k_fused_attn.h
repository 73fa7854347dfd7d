// Attention half of the temporal-block kernel (k_fused_block.h): layout notes, head-group helpers
// and the cooperative slice-in.  The chain is
//   slice window -> GroupNorm -> proj_in -> LN1 (+ frame embedding) -> q, k, v
//   -> per-position attention over the F frames.
//
// One wavefront carries 32 token columns = TP = floor(32/F) whole positions x F frames (columns
// beyond TP*F are padding), so every sequence the attention needs sits inside one wavefront and
// the chain runs in MFMA result layout as in k_fused.h:
//   q, k   result layout (lane = token, registers = feature columns) is already the operand
//          layout of S^T = K Q^T (keys as rows, queries as columns);
//   v      is formed transposed (activations as the row operand, W_v fragments as columns), which
//          makes its result registers the row operand V^T of O^T = V^T P^T;
//   P^T    the softmax result registers (lane = query, registers = keys) are the column operand.
// Heads are handled in groups whose width lcm(dim_head, 32) is a whole number of 32-column
// blocks; inside a group a head's columns are selected by zeroing the other 8-column halves of
// the q operand and by picking result quads (dim_head % 8 == 0 keeps both static).
// Scores never leave registers; the softmax runs per lane over its 16 key registers plus one
// cross-lane exchange (lane ^ 32).
#pragma once
#include "k_fused.h"

namespace si {

__host__ __device__ constexpr int gcd_int(int a, int b) { return b == 0 ? a : gcd_int(b, a % b); }
__host__ __device__ constexpr int lcm_int(int a, int b) { return a / gcd_int(a, b) * b; }

constexpr int kAttnMaxStats = 896;  // F * G entries per batch entry held in LDS

// Cooperative slice-in of one workgroup tile (see temporal_block_kernel).  NPOS consecutive sequences
// (b, position) starting at seq_wg; xs row of (sequence j, frame f) = (j / TP) * 32 + (j % TP) * F + f.
template <int U, int D, int XLD>
__device__ __forceinline__ void stage_window(const bf16* __restrict__ x, unsigned short* xs, const float2* t_stats,
                                             const float* t_gng, const float* t_gnb, const Window& w, int64_t seq_wg,
                                             int64_t nseq, int b_first, int TP, int NPOS, int tid) {
  const int F = w.F;
  const int runs = NPOS / U, pairs = runs * F;  // <= 128
  int PP = 1;
  while (PP < pairs) PP *= 2;
  const int CL = 256 / PP;  // channel lanes
  const int pair = tid % PP, cl = tid / PP;
  const int run = pair % runs, f = pair / runs;
  const int j0 = run * U;
  const int64_t seq = seq_wg + j0;
  if (pair >= pairs || seq >= nseq) return;  // runs never straddle the end: nseq % U == 0 when U > 1
  const int b = (int)seq / w.Pw, pl = (int)seq % w.Pw;  // sequences of a window fit 31 bits
  const int ng = w.C / w.G;
  const float2* st = t_stats + (b - b_first) * kAttnMaxStats + f * w.G;
  const bf16* xp = x + (((int64_t)b * w.C + cl) * F + f) * w.P + w.p0 + pl;
  const int64_t cstep = (int64_t)CL * F * w.P;
  int rows[U];
#pragma unroll
  for (int u = 0; u < U; ++u) rows[u] = ((j0 + u) / TP) * 32 + ((j0 + u) % TP) * F + f;
  int grp = cl / ng, left = ng - (cl % ng);
  constexpr int BATCH = 8;
  for (int c0 = cl; c0 < D; c0 += BATCH * CL) {
    uint2 raw[BATCH];
#pragma unroll
    for (int k = 0; k < BATCH; ++k) {
      if (c0 + k * CL < D) {
        if constexpr (U == 4) raw[k] = *reinterpret_cast<const uint2*>(xp + k * cstep);
        else raw[k].x = xp[k * cstep].v;
      }
    }
#pragma unroll
    for (int k = 0; k < BATCH; ++k) {
      const int c = c0 + k * CL;
      if (c < D) {
        const float2 ms = st[grp];
        const float sc = ms.y * t_gng[c], sh = t_gnb[c] - ms.x * sc;
        if constexpr (U == 4) {
          xs[rows[0] * XLD + c] = float_to_bf16_bits(fmaf(__uint_as_float(raw[k].x << 16), sc, sh));
          xs[rows[1] * XLD + c] = float_to_bf16_bits(fmaf(__uint_as_float(raw[k].x & 0xffff0000u), sc, sh));
          xs[rows[2] * XLD + c] = float_to_bf16_bits(fmaf(__uint_as_float(raw[k].y << 16), sc, sh));
          xs[rows[3] * XLD + c] = float_to_bf16_bits(fmaf(__uint_as_float(raw[k].y & 0xffff0000u), sc, sh));
        } else {
          xs[rows[0] * XLD + c] = float_to_bf16_bits(fmaf(bf16_bits_to_float((unsigned short)raw[k].x), sc, sh));
        }
        left -= CL;
        while (left <= 0) {
          ++grp;
          left += ng;
        }
      }
    }
    xp += BATCH * cstep;
  }
}

}  // namespace si
