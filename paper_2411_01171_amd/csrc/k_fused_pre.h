// Register-resident kernel in front of a spatial block's self-attention (D = 32*NB = C, bf16
// storage, frames that are whole 128-token workgroup tiles):
//   slice window -> GroupNorm -> proj_in -> h;  LN1(h) -> q (pre-scaled), k rows and V transposed.
// Same scheme as k_fused.h: tokens are the MFMA columns, one wavefront carries 32 tokens, the
// weights arrive as a fragment stream through the LDS ring.  The x operand is gathered straight
// from the feature tensor: for one channel the 32 tokens of a wavefront are 64 contiguous bytes.
// proj_in runs on fp16 operands (the normalised input is bounded; three more significand bits than
// bf16), everything behind LN1 on bf16.  q, k and v leave as the MFMA fragments that the attention
// kernel consumes (attn_mfma_kernel, FRAGIN): a result block's register halves, packed to bf16, are
// such fragments as they stand -- for v with the operands swapped (activations as the row operand),
// which yields V^T.  Every store of a wavefront is one contiguous KiB.
#pragma once
#include "k_fused.h"

namespace si {

struct SpatialPreArgs {
  const bf16* x;
  const float* stats;     // (mean, rstd) per (b, f, group)
  const bf16 *gn_g, *gn_b, *b_in, *ln_g, *ln_b;
  const u32x4_t* stream;  // W_in blocks (fp16), then W_q, W_k, W_v blocks: 4 * NB sub-chunks
  float* h;               // residual stream, workgroup-tile order (h_tile_index)
  u32x4_t* qf;            // q * qscale as fragments: [(sequence, head)][32-query tile][k-step 0..3][lane]
  u32x4_t* kvf;           // k and v^T as fragments: [(sequence, head)][64-key stage][16][lane], the attention
                          // kernel's stage order (attn_mfma_kernel, FRAGIN)
  int64_t M;              // tokens of the window, a multiple of 128; sequence (b, f) = rows (b*Fw + f)*Pw + i
  float ln_eps, qscale;
  Window win;             // p0 == 0, Pw == P, P % 128 == 0
};

template <int NB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void spatial_pre_kernel(SpatialPreArgs a) {
  constexpr int D = 32 * NB, SUB = 2 * NB;
  constexpr int NSLOT = kRingSlots, FIFO = NB;
  constexpr int TOTAL_SUB = 4 * NB;
  static_assert(NB % 2 == 0, "NB must be even");
  typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
  __shared__ u32x4_t ring[NSLOT][SUB * kWave];
  __shared__ float t_sc[D], t_sh[D], t_bin[D], t_g[D], t_b[D];

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int r = lane % 32, g = lane / 32;
  const Window& w = a.win;
  const int64_t m0 = (int64_t)blockIdx.x * 128;
  const int seq = (int)m0 / w.Pw, b = seq / w.Fw, f = w.f0 + seq % w.Fw;  // window tokens fit 31 bits
  const int key0 = (int)m0 % w.Pw + wave * 32;  // first position of this wavefront inside its frame

  {  // GroupNorm of this frame as one multiply-add per channel, and the other per-channel tables
    const int ng = w.C / w.G;
    const float* st = a.stats + ((int64_t)b * w.F + f) * w.G * 2;
    for (int i = tid; i < D; i += 256) {
      const float mean = st[(i / ng) * 2], rstd = st[(i / ng) * 2 + 1];
      const float sc = rstd * param_or(a.gn_g, i, 1.f);
      t_sc[i] = sc;
      t_sh[i] = param_or(a.gn_b, i, 0.f) - mean * sc;
      t_bin[i] = param_or(a.b_in, i, 0.f);
      t_g[i] = param_or(a.ln_g, i, 1.f);
      t_b[i] = param_or(a.ln_b, i, 0.f);
    }
  }

  using Pipe = WeightPipe<SUB>;
  const int64_t pitch = stream_pitch_u4(TOTAL_SUB);
  const unsigned pipe_voff = Pipe::pipe_voff(lane, wave, pitch);
  const int pipe_wave = __builtin_amdgcn_readfirstlane(wave);
  int cur = 0;
#pragma unroll
  for (int i = 0; i < NSLOT - 1; ++i) Pipe::issue(a.stream, ring[0], i, TOTAL_SUB, pitch, pipe_voff, pipe_wave);

  // ---- this lane's token as fp16 column operands: k-step s holds channels 16s + frag_k(g, e)
  half8_t xop[SUB];
  {
    const int64_t cs = (int64_t)w.F * w.P;
    const bf16* xp = a.x + ((int64_t)b * w.C * w.F + f) * w.P + w.p0 + key0 + r;
    unsigned short raw[SUB][8];
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) raw[s][e] = xp[(int64_t)(16 * s + frag_k(g, e)) * cs].v;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the gathers and the first sub-chunks
    __syncthreads();                     // tables and the first three sub-chunks are in LDS
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int c = 16 * s + frag_k(g, e);
        const float v = fmaf(bf16_bits_to_float(raw[s][e]), t_sc[c], t_sh[c]);
        xop[s][e] = (_Float16)__builtin_amdgcn_fmed3f(v, -65504.f, 65504.f);
      }
  }

  bf16x8_t fifo[FIFO];
#pragma unroll
  for (int i = 0; i < FIFO; ++i) fifo[i] = __builtin_bit_cast(bf16x8_t, ring[0][i * kWave + lane]);

#define SI_STEP_OPEN()                                                                      \
  __builtin_amdgcn_sched_barrier(0);                                                        \
  Pipe::issue(a.stream, ring[0], cur + NSLOT - 1, TOTAL_SUB, pitch, pipe_voff, pipe_wave);  \
  const u32x4_t* slot_c = ring[cur % NSLOT];                                                \
  const u32x4_t* slot_n = ring[(cur + 1) % NSLOT];                                          \
  (void)slot_c; (void)slot_n
#define SI_STEP_CLOSE()                          \
  __builtin_amdgcn_sched_barrier(0);             \
  Pipe::template wait_step<0>(cur, TOTAL_SUB);   \
  ++cur;                                         \
  SI_RING_BARRIER()
#define SI_FRAG(f) fifo[(f) % FIFO]
#define SI_REFILL(f)                                                                                 \
  fifo[(f) % FIFO] = __builtin_bit_cast(bf16x8_t, (f) < FIFO ? slot_c[((f) + FIFO) * kWave + lane]   \
                                                             : slot_n[((f)-FIFO) * kWave + lane])

  // ---- proj_in: h[nb][4q + j] = channel 32nb + 8q + 4g + j of this lane's token
  f32x16_t hacc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int e = 0; e < 16; ++e) hacc[nb][e] = 0.f;
    {
      SI_STEP_OPEN();
#pragma unroll
      for (int s = 0; s < SUB; ++s) {
        hacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, SI_FRAG(s)), xop[s], hacc[nb], 0, 0, 0);
        SI_REFILL(s);
        __builtin_amdgcn_sched_barrier(0);
      }
      SI_STEP_CLOSE();
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float4 v;
      v.x = hacc[nb][4 * q + 0] += t_bin[32 * nb + 8 * q + 4 * g + 0];
      v.y = hacc[nb][4 * q + 1] += t_bin[32 * nb + 8 * q + 4 * g + 1];
      v.z = hacc[nb][4 * q + 2] += t_bin[32 * nb + 8 * q + 4 * g + 2];
      v.w = hacc[nb][4 * q + 3] += t_bin[32 * nb + 8 * q + 4 * g + 3];
      reinterpret_cast<float4*>(a.h)[h_tile_index<NB>(blockIdx.x, nb, q, wave, lane)] = v;
    }
  }

  // ---- LN1 over the row (this lane holds half of it, lane ^ 32 the other half) -> bf16 operands
  bf16x8_t aop[SUB];
  {
    float s = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += hacc[nb][e];
    s += __shfl_xor(s, 32, kWave);
    const float mean = s * (1.0f / D);
    float qv = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float dlt = hacc[nb][e] - mean;
        qv = fmaf(dlt, dlt, qv);
      }
    qv += __shfl_xor(qv, 32, kWave);
    const float rstd = rsqrtf(qv * (1.0f / D) + a.ln_eps);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int n = 32 * nb + 16 * hf + frag_k(g, e);
          v[e] = (hacc[nb][8 * hf + e] - mean) * rstd * t_g[n] + t_b[n];
        }
        aop[2 * nb + hf] = to_operand(v);
      }
  }

  // ---- q (scaled) and k: a result block's two register halves are two fragments as they are (lane =
  // token, elements = channels 16 ks + frag_k(g, e) of the head) -- one contiguous KiB per store
  constexpr int NH = D / 64;
  const int tile = key0 / 32, tiles = w.Pw / 32;  // this wavefront's 32 tokens inside their sequence
  u32x4_t* const qdst = a.qf + ((int64_t)seq * NH * tiles + tile) * 4 * kWave + lane;
  u32x4_t* const kvdst = a.kvf + (((int64_t)seq * NH * (tiles / 2) + tile / 2) * 16 + 4 * (tile % 2)) * kWave + lane;
#pragma unroll
  for (int blk = 0; blk < 2 * NB; ++blk) {
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    {
      SI_STEP_OPEN();
#pragma unroll
      for (int s = 0; s < SUB; ++s) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), aop[s], acc, 0, 0, 0);
        SI_REFILL(s);
        __builtin_amdgcn_sched_barrier(0);
      }
      SI_STEP_CLOSE();
    }
    const float sc = blk < NB ? a.qscale : 1.f;
    const int nb = blk % NB, hd = nb / 2;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = acc[8 * hf + e] * sc;
      const u32x4_t o = __builtin_bit_cast(u32x4_t, to_operand(v));
      const int ks = 2 * (nb % 2) + hf;
      if (blk < NB) qdst[((int64_t)hd * tiles * 4 + ks) * kWave] = o;
      else kvdst[((int64_t)hd * (tiles / 2) * 16 + ks) * kWave] = o;
    }
  }

  // ---- V^T: activations as the row operand, so lane = channel 32nb + r, register 4q + j = token 8q + 4g + j:
  // the two register halves are the V^T fragments of 16-key steps 0 and 1 (keys 16 t + frag_k(g, e))
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    {
      SI_STEP_OPEN();
#pragma unroll
      for (int s = 0; s < SUB; ++s) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[s], SI_FRAG(s), acc, 0, 0, 0);
        SI_REFILL(s);
        __builtin_amdgcn_sched_barrier(0);
      }
      SI_STEP_CLOSE();
    }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = acc[8 * hf + e];
      kvdst[((int64_t)(nb / 2) * (tiles / 2) * 16 + 8 + 2 * (nb % 2) + hf) * kWave] = __builtin_bit_cast(u32x4_t, to_operand(v));
    }
  }
#undef SI_REFILL
#undef SI_FRAG
#undef SI_STEP_CLOSE
#undef SI_STEP_OPEN
}

}  // namespace si
