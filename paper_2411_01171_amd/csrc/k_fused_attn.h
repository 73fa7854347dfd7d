// Register-resident attention half of a temporal block (bf16, C == D = 32*NB <= 320):
//   slice window -> GroupNorm -> proj_in -> (h0 to memory) -> LN1 (+ frame embedding)
//   -> q, k, v -> per-position attention over the F frames -> o (to memory).
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

struct AttnHalfArgs {
  const bf16* x;        // [B, C, F, H*W]
  const float* stats;   // [B, F, G, 2] GroupNorm mean / rstd
  const bf16 *gn_g, *gn_b, *b_in, *ln_g, *ln_b;
  const float* pe;      // [F, D] frame embedding or NULL
  const u32x4_t* stream;  // W_in blocks, then per head group: q blocks, k blocks, v blocks
  float* h0;            // out: [M, D] residual stream after proj_in
  bf16* o;              // out: [M, D] attention output, heads concatenated
  float ln_eps, scale;
  Window win;           // temporal window: all F frames, positions [p0, p0 + Pw)
};

constexpr int kAttnMaxStats = 896;  // F * G entries per batch entry held in LDS

// Cooperative slice-in of one workgroup tile (see attn_half_kernel).  NPOS consecutive sequences
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
  const int b = (int)(seq / w.Pw), pl = (int)(seq % w.Pw);
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

template <int NB, int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_half_kernel(AttnHalfArgs a) {
  constexpr int D = 32 * NB, SUB = 2 * NB, NSLOT = kRingSlots, FIFO = NB;
  constexpr int GW = lcm_int(DH, 32);        // columns per head group
  constexpr int NBG = GW / 32, HG = GW / DH;  // blocks / heads per group
  constexpr int NG = D / GW;
  constexpr int TOTAL_SUB = NB + 3 * NB;
  constexpr int XLD = D + 8;  // padded row of the staged x tile (bf16 elements)
  static_assert(NB % 2 == 0 && D % GW == 0 && DH % 8 == 0, "shape");
  constexpr int SLOT_BYTES = SUB * kWave * 16, XS_BYTES = 128 * XLD * 2;
  // ring slots 0 and 1 are loaded while the staged x tile is in use; the tile shares LDS with slots 2, 3
  constexpr int TAIL_BYTES = 2 * SLOT_BYTES > XS_BYTES ? 2 * SLOT_BYTES : XS_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char arena[2 * SLOT_BYTES + TAIL_BYTES];
  __shared__ float2 t_stats[2][kAttnMaxStats];
  __shared__ __attribute__((aligned(16))) float t_gng[D], t_gnb[D], t_bin[D], t_lg[D], t_lb[D];
  u32x4_t(*ring)[SUB * kWave] = reinterpret_cast<u32x4_t(*)[SUB * kWave]>(arena);
  unsigned short* xs = reinterpret_cast<unsigned short*>(arena + 2 * SLOT_BYTES);

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int tcol = lane % 32, g = lane / 32;
  const Window& w = a.win;
  const int F = w.F, TP = 32 / F, NPOS = 4 * TP;  // positions per workgroup
  const int64_t nseq = (int64_t)w.B * w.Pw;       // sequences (b, position) of the window
  // Eight consecutive tiles share the cache lines of x (runs of 64 positions).  Workgroups are
  // handed to the 8 XCDs round-robin, so tile = f(blockIdx) is chosen to put such a run of tiles
  // on one XCD (one L2), in consecutive dispatch rounds: tile = 64*(b/64) + 8*(b%8) + (b/8)%8.
  const unsigned bid = blockIdx.x, full = gridDim.x / 64 * 64;
  const unsigned tile = bid < full ? (bid / 64) * 64 + (bid % 8) * 8 + (bid / 8) % 8 : bid;
  const int64_t seq_wg = (int64_t)tile * NPOS;

  // this lane's token: sequence, frame, row of the window's token order m = (b*F + f)*Pw + pl
  const int my_pp = tcol / F, my_f = tcol % F;
  const int64_t my_seq = seq_wg + wave * TP + my_pp;
  const bool live = tcol < TP * F && my_seq < nseq;
  const int my_b = live ? (int)(my_seq / w.Pw) : 0, my_pl = live ? (int)(my_seq % w.Pw) : 0;
  const int64_t my_m = ((int64_t)my_b * F + my_f) * w.Pw + my_pl;

  // ---- weight stream (see WeightPipe): sub-chunks 0 and 1 now, sub-chunk 2 once the x tile has left LDS
  using Pipe = WeightPipe<SUB>;
  const int64_t pitch = stream_pitch_u4(TOTAL_SUB);
  const unsigned pipe_voff = Pipe::pipe_voff(lane, wave, pitch);
  const int pipe_wave = __builtin_amdgcn_readfirstlane(wave);
  int cur = 0;
  Pipe::issue(a.stream, ring[0], 0, TOTAL_SUB, pitch, pipe_voff, pipe_wave);
  Pipe::issue(a.stream, ring[0], 1, TOTAL_SUB, pitch, pipe_voff, pipe_wave);

  // ---- tables; the staged tile starts as zeros (padding rows and columns stay zero)
  const int b_first = (int)(seq_wg / w.Pw);
  for (int i = tid; i < D; i += 256) {
    t_gng[i] = param_or(a.gn_g, i, 1.f);
    t_gnb[i] = param_or(a.gn_b, i, 0.f);
    t_bin[i] = param_or(a.b_in, i, 0.f);
    t_lg[i] = param_or(a.ln_g, i, 1.f);
    t_lb[i] = param_or(a.ln_b, i, 0.f);
  }
  for (int i = tid; i < 2 * F * w.G; i += 256) {
    const int bs = i / (F * w.G), r = i % (F * w.G);
    const int bb = b_first + bs;
    float2 st = make_float2(0.f, 0.f);
    if (bb < w.B) st = *reinterpret_cast<const float2*>(a.stats + ((int64_t)bb * F * w.G + r) * 2);
    t_stats[bs][r] = st;
  }
  for (int i = tid; i < XS_BYTES / 16; i += 256) reinterpret_cast<u32x4_t*>(xs)[i] = u32x4_t{0, 0, 0, 0};
  __syncthreads();

  // ---- slice-in: x[b, c, f, p0 + pl] -> GroupNorm -> xs[row][c].  A thread owns one (frame,
  // run of U consecutive positions) pair and walks the channels with stride 256 / PP; loads are
  // issued in batches ahead of their use.  U = 4 (8-byte loads) when rows, window start and frame
  // size are multiples of 4 positions, else U = 1.
  if ((w.Pw % 4 == 0) && (w.p0 % 4 == 0) && (w.P % 4 == 0))
    stage_window<4, D, XLD>(a.x, xs, t_stats[0], t_gng, t_gnb, w, seq_wg, nseq, b_first, TP, NPOS, tid);
  else
    stage_window<1, D, XLD>(a.x, xs, t_stats[0], t_gng, t_gnb, w, seq_wg, nseq, b_first, TP, NPOS, tid);
  __syncthreads();

  // ---- this wavefront's GroupNorm'ed tokens as column operands
  bf16x8_t aop[SUB];
  {
    const unsigned short* xrow = xs + (wave * 32 + tcol) * XLD;
#pragma unroll
    for (int s = 0; s < SUB; ++s) {
      const uint2 lo = *reinterpret_cast<const uint2*>(xrow + 16 * s + 4 * g);
      const uint2 hi = *reinterpret_cast<const uint2*>(xrow + 16 * s + 8 + 4 * g);
      u32x4_t u;
      u.x = lo.x; u.y = lo.y; u.z = hi.x; u.w = hi.y;
      aop[s] = __builtin_bit_cast(bf16x8_t, u);
    }
  }
  __syncthreads();  // every wavefront has its operands: the tile's LDS becomes ring slots 2 and 3
  Pipe::issue(a.stream, ring[0], 2, TOTAL_SUB, pitch, pipe_voff, pipe_wave);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __syncthreads();

  bf16x8_t fifo[FIFO];
#pragma unroll
  for (int i = 0; i < FIFO; ++i) fifo[i] = __builtin_bit_cast(bf16x8_t, ring[0][i * kWave + lane]);

#define SI_STEP_OPEN()                                                           \
  __builtin_amdgcn_sched_barrier(0);                                             \
  Pipe::issue(a.stream, ring[0], cur + 3, TOTAL_SUB, pitch, pipe_voff, pipe_wave);         \
  const u32x4_t* slot_c = ring[cur % NSLOT];                                     \
  const u32x4_t* slot_n = ring[(cur + 1) % NSLOT];                               \
  (void)slot_c; (void)slot_n
#define SI_STEP_CLOSE()                                                          \
  __builtin_amdgcn_sched_barrier(0);                                             \
  Pipe::template wait_step<0>(cur, TOTAL_SUB);                                   \
  ++cur;                                                                         \
  __syncthreads()
#define SI_FRAG(f) fifo[(f) % FIFO]
#define SI_REFILL(f)                                                                                 \
  fifo[(f) % FIFO] = __builtin_bit_cast(bf16x8_t, (f) < FIFO ? slot_c[((f) + FIFO) * kWave + lane]   \
                                                             : slot_n[((f)-FIFO) * kWave + lane])
  // one 32-column block: weights as rows (result: lane = token) or as columns (result: lane = column)
#define SI_BLOCK_WROWS(ACC)                                                                 \
  {                                                                                         \
    SI_STEP_OPEN();                                                                         \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) ACC[e] = 0.f;                            \
    _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                       \
      ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), aop[s], ACC, 0, 0, 0);      \
      SI_REFILL(s);                                                                         \
      __builtin_amdgcn_sched_barrier(0);                                                    \
    }                                                                                       \
    SI_STEP_CLOSE();                                                                        \
  }
#define SI_BLOCK_WCOLS(ACC)                                                                 \
  {                                                                                         \
    SI_STEP_OPEN();                                                                         \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) ACC[e] = 0.f;                            \
    _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                       \
      ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[s], SI_FRAG(s), ACC, 0, 0, 0);      \
      SI_REFILL(s);                                                                         \
      __builtin_amdgcn_sched_barrier(0);                                                    \
    }                                                                                       \
    SI_STEP_CLOSE();                                                                        \
  }

  // ---- proj_in, h0 to memory
  f32x16_t hacc[NB];
#define SI_PROJ_IN_BLOCK(nb)                                                                         \
  {                                                                                                  \
    SI_BLOCK_WROWS(hacc[nb])                                                                         \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                  \
      const float4 bb = *reinterpret_cast<const float4*>(&t_bin[32 * (nb) + 8 * q + 4 * g]);         \
      hacc[nb][4 * q + 0] += bb.x; hacc[nb][4 * q + 1] += bb.y;                                      \
      hacc[nb][4 * q + 2] += bb.z; hacc[nb][4 * q + 3] += bb.w;                                      \
      if (live)                                                                                      \
        *reinterpret_cast<float4*>(a.h0 + my_m * D + 32 * (nb) + 8 * q + 4 * g) =                    \
            make_float4(hacc[nb][4 * q + 0], hacc[nb][4 * q + 1], hacc[nb][4 * q + 2], hacc[nb][4 * q + 3]); \
    }                                                                                                \
  }
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) SI_PROJ_IN_BLOCK(nb)
#undef SI_PROJ_IN_BLOCK

  // ---- LN1 (+ frame embedding): aop becomes its output
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
    const float* perow = a.pe ? a.pe + (int64_t)my_f * D : nullptr;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float v[8];
#pragma unroll
        for (int e4 = 0; e4 < 8; e4 += 4) {
          const int n = 32 * nb + 16 * hf + frag_k(g, e4);  // four consecutive columns
          const float4 gg = *reinterpret_cast<const float4*>(&t_lg[n]);
          const float4 bb = *reinterpret_cast<const float4*>(&t_lb[n]);
          float4 pp = make_float4(0.f, 0.f, 0.f, 0.f);
          if (perow) pp = *reinterpret_cast<const float4*>(perow + n);
          v[e4 + 0] = (hacc[nb][8 * hf + e4 + 0] - mean) * rstd * gg.x + bb.x + pp.x;
          v[e4 + 1] = (hacc[nb][8 * hf + e4 + 1] - mean) * rstd * gg.y + bb.y + pp.y;
          v[e4 + 2] = (hacc[nb][8 * hf + e4 + 2] - mean) * rstd * gg.z + bb.z + pp.z;
          v[e4 + 3] = (hacc[nb][8 * hf + e4 + 3] - mean) * rstd * gg.w + bb.w + pp.w;
        }
        aop[2 * nb + hf] = to_operand(v);
      }
  }

  // ---- attention.  Key validity per result register: key row i = 8q + 4g + j of the 32 token
  // columns is a key of this lane's query iff both belong to the same position and i < TP*F.
  unsigned kvalid = 0;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = 8 * (v / 4) + 4 * g + (v % 4);
    if (i < TP * F && i / F == my_pp) kvalid |= 1u << v;
  }
  const float sl2 = a.scale * 1.4426950408889634f;  // scores are exponentiated in base 2

  // ---- groups of heads
  {
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      bf16x8_t qop[2 * NBG], kop[2 * NBG], vop[2 * NBG];
#pragma unroll
      for (int kind = 0; kind < 3; ++kind) {
#pragma unroll
        for (int blk = 0; blk < NBG; ++blk) {
          f32x16_t acc;
          if (kind < 2) SI_BLOCK_WROWS(acc) else SI_BLOCK_WCOLS(acc)
          float lo[8], hi[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            lo[e] = acc[e];
            hi[e] = acc[8 + e];
          }
          if (kind == 0) {
            qop[2 * blk] = to_operand(lo);
            qop[2 * blk + 1] = to_operand(hi);
          } else if (kind == 1) {
            kop[2 * blk] = to_operand(lo);
            kop[2 * blk + 1] = to_operand(hi);
          } else {
            vop[2 * blk] = to_operand(lo);
            vop[2 * blk + 1] = to_operand(hi);
          }
        }
      }
#pragma unroll
      for (int hh = 0; hh < HG; ++hh) {
        const int c0 = hh * DH, c1 = c0 + DH;  // head columns inside the group
        // S^T[key, query] over the head's columns; 8-column halves of other heads are zeroed in q
        f32x16_t sc;
#pragma unroll
        for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
        for (int s = 0; s < 2 * NBG; ++s) {
          const bool in0 = 16 * s >= c0 && 16 * s + 8 <= c1;       // columns [16s, 16s+8)
          const bool in1 = 16 * s + 8 >= c0 && 16 * s + 16 <= c1;  // columns [16s+8, 16s+16)
          if (in0 || in1) {
            u32x4_t qm = __builtin_bit_cast(u32x4_t, qop[s]);
            if (!in0) { qm.x = 0; qm.y = 0; }
            if (!in1) { qm.z = 0; qm.w = 0; }
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s], __builtin_bit_cast(bf16x8_t, qm), sc, 0, 0, 0);
          }
        }
        // softmax over this query's keys (16 registers here, 16 in lane ^ 32)
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kvalid & (1u << v)) mx = fmaxf(mx, sc[v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        if (mx == -INFINITY) mx = 0.f;  // padding column: no keys
        float pr[16], sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          pr[v] = (kvalid & (1u << v)) ? __builtin_amdgcn_exp2f((sc[v] - mx) * sl2) : 0.f;
          sum += pr[v];
        }
        sum += __shfl_xor(sum, 32, kWave);
        const float inv = sum > 0.f ? 1.0f / sum : 0.f;
        bf16x8_t pop[2];
        pop[0] = to_operand(&pr[0]);
        pop[1] = to_operand(&pr[8]);
        // O^T[column, query] for the blocks the head touches; keep the head's quads
#pragma unroll
        for (int blk = 0; blk < NBG; ++blk) {
          if (32 * blk < c1 && 32 * blk + 32 > c0) {
            f32x16_t ot;
#pragma unroll
            for (int e = 0; e < 16; ++e) ot[e] = 0.f;
            ot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[2 * blk], pop[0], ot, 0, 0, 0);
            ot = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[2 * blk + 1], pop[1], ot, 0, 0, 0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int col = 32 * blk + 8 * q;  // quad q: columns [col, col+8) of the group
              if (col >= c0 && col < c1 && live) {
                // attention output, heads concatenated: o[m][gi*GW + 32 blk + 8q + 4g + j]
                uint2 pk;
                pk.x = pack_bf16x2(ot[4 * q + 0] * inv, ot[4 * q + 1] * inv);
                pk.y = pack_bf16x2(ot[4 * q + 2] * inv, ot[4 * q + 3] * inv);
                *reinterpret_cast<uint2*>(a.o + my_m * D + gi * GW + col + 4 * g) = pk;
              }
            }
          }
        }
      }
    }
  }
#undef SI_BLOCK_WCOLS
#undef SI_BLOCK_WROWS
#undef SI_REFILL
#undef SI_FRAG
#undef SI_STEP_CLOSE
#undef SI_STEP_OPEN
}

}  // namespace si
