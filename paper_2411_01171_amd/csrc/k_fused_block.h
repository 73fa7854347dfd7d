// One kernel per slice window for temporal blocks (bf16, C == D = 32*NB <= 320):
//   slice window -> GroupNorm -> proj_in -> LN1 (+ frame embedding) -> q, k, v -> per-position
//   attention over the F frames -> out-projection + residual -> LN3 -> GEGLU FFN + residual ->
//   proj_out -> + x -> out window.
//
// It chains the attention half (k_fused_attn.h) and the FFN half (k_fused.h) in one wavefront
// program: the attention output stays in registers as the column operand of the out-projection,
// and the only activation that leaves the registers is the residual stream after proj_in, parked
// in a per-workgroup scratch in register-image order (1 KiB per store instruction, read back by
// the same lanes) while the attention needs the registers.  One wavefront = floor(32/F) whole
// positions x F frames; see the two halves for the layout arguments.
//
// Slice-out: a workgroup owns NPOS = 4*floor(32/F) consecutive positions of every frame.  Each
// proj_out block (32 channels) goes through an LDS patch [channel][frame][position] so that one
// lane handles the NPOS-position run of one (channel, frame): one vector load of x, one vector
// store of out.  Runs of consecutive tiles complete the cache lines; the XCD-aware tile order keeps
// such runs on one L2.
#pragma once
#include "k_fused_attn.h"

namespace si {

struct TemporalBlockArgs {
  const bf16* x;        // [B, C, F, H*W]
  bf16* out;            // [B, C, F, H*W]
  const float* stats;   // [B, F, G, 2] GroupNorm mean / rstd
  const bf16 *gn_g, *gn_b, *b_in, *ln1_g, *ln1_b, *b_o, *ln3_g, *ln3_b, *b1, *b2, *b_out;
  const float* pe;      // [F, D] frame embedding or NULL
  const u32x4_t* stream;  // W_in blocks; per head group q, k, v blocks; W_o blocks; FFN; W_out blocks
  float* hpark;         // scratch: gridDim.x * 128 * D floats.  SPLIT: the residual stream after proj_in of the
                        // window's tokens m = (b*F + f)*Pw + position in the FFN-half kernel's workgroup-tile
                        // order (h_tile_index; whole 128-token tiles) + 4 KiB that idle lanes write to
  bf16* o_rows;         // SPLIT: the attention output as that kernel's operand fragments [m / 32][k-step][lane]
  float ln_eps, scale;
  Window win;           // temporal window: all F frames, positions [p0, p0 + Pw)
};

// SPLIT: the kernel ends behind the attention and leaves the residual stream and the attention
// output as token rows; ffn_half_kernel (k_fused.h) takes the window on from there with its
// wavefronts' 32 columns all in use -- worth it when F leaves many of this kernel's 32 columns per
// wavefront empty (F = 25: 7 of 32), because three quarters of the window's MFMAs lie behind the cut.
template <int NB, int DH, bool SPLIT = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void temporal_block_kernel(TemporalBlockArgs a) {
  constexpr int D = 32 * NB, SUB = 2 * NB, NC = 4 * NB, NSLOT = kRingSlots, FIFO = NB;
  constexpr int GW = lcm_int(DH, 32);        // columns per head group
  constexpr int NBG = GW / 32, HG = GW / DH;  // blocks / heads per group
  constexpr int NG = D / GW;
  constexpr int TOTAL_SUB = SPLIT ? 4 * NB : 4 * NB + NB + 3 * NC + NB;
  constexpr int XLD = D + 8;  // padded row of the staged x tile (bf16 elements)
  static_assert(NB % 2 == 0 && D % GW == 0 && DH % 8 == 0, "shape");
  constexpr int SLOT_BYTES = SUB * kWave * 16, XS_BYTES = 128 * XLD * 2;
  constexpr int PATCH_LD = 128 + 4, PATCH_BYTES = 2 * 32 * PATCH_LD * 4;  // two slice-out patches
  // ring slots 0 and 1 are loaded while the staged x tile is in use; the tile shares LDS with slots
  // 2, 3 and (behind them) the slice-out patches
  constexpr int TAIL_BYTES = 2 * SLOT_BYTES + PATCH_BYTES > XS_BYTES ? 2 * SLOT_BYTES + PATCH_BYTES : XS_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char arena[2 * SLOT_BYTES + TAIL_BYTES];
  __shared__ float2 t_stats[2][kAttnMaxStats];
  __shared__ __attribute__((aligned(16))) float t_gng[D], t_gnb[D], t_bin[D], t_lg[D], t_lb[D];
  __shared__ __attribute__((aligned(16))) float t_g[D], t_b[D], t_b2[D], t_bout[D], t_bo[D];
  __shared__ __attribute__((aligned(16))) float t_b1[8 * D];
  u32x4_t(*ring)[SUB * kWave] = reinterpret_cast<u32x4_t(*)[SUB * kWave]>(arena);
  unsigned short* xs = reinterpret_cast<unsigned short*>(arena + 2 * SLOT_BYTES);
  float(*patch)[32][PATCH_LD] = reinterpret_cast<float(*)[32][PATCH_LD]>(arena + 4 * SLOT_BYTES);

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
  // SPLIT: row of this lane's token, or (padding column, sequence past the end) a dump row
  const int64_t my_seq = seq_wg + wave * TP + my_pp;
  const bool row_live = tcol < TP * F && my_seq < nseq;
  const int my_si = (int)my_seq;  // sequences of a window fit 31 bits: 32-bit divisions throughout this kernel
  const int64_t my_row = row_live ? ((int64_t)(my_si / w.Pw) * F + my_f) * w.Pw + my_si % w.Pw : 0;

  // ---- weight stream (see WeightPipe): sub-chunks 0 and 1 now, sub-chunk 2 once the x tile has left LDS
  using Pipe = WeightPipe<SUB>;
  const int64_t pitch = stream_pitch_u4(TOTAL_SUB);
  const unsigned pipe_voff = Pipe::pipe_voff(lane, wave, pitch);
  const int pipe_wave = __builtin_amdgcn_readfirstlane(wave);
  int cur = 0;
  Pipe::issue(a.stream, ring[0], 0, TOTAL_SUB, pitch, pipe_voff, pipe_wave);
  Pipe::issue(a.stream, ring[0], 1, TOTAL_SUB, pitch, pipe_voff, pipe_wave);

  // ---- tables; the staged tile starts as zeros (padding rows and columns stay zero)
  const int b_first = (int)seq_wg / w.Pw;
  for (int i = tid; i < D; i += 256) {
    t_gng[i] = param_or(a.gn_g, i, 1.f);
    t_gnb[i] = param_or(a.gn_b, i, 0.f);
    t_bin[i] = param_or(a.b_in, i, 0.f);
    t_lg[i] = param_or(a.ln1_g, i, 1.f);
    t_lb[i] = param_or(a.ln1_b, i, 0.f);
    t_g[i] = param_or(a.ln3_g, i, 1.f);
    t_b[i] = param_or(a.ln3_b, i, 0.f);
    t_b2[i] = param_or(a.b2, i, 0.f);
    t_bout[i] = param_or(a.b_out, i, 0.f);
    t_bo[i] = param_or(a.b_o, i, 0.f);
  }
  for (int i = tid; i < 8 * D; i += 256) t_b1[i] = param_or(a.b1, i, 0.f);
  for (int i = tid; i < 2 * F * w.G; i += 256) {
    const int bs = i / (F * w.G), r = i % (F * w.G);
    const int bb = b_first + bs;
    float2 st = make_float2(0.f, 0.f);
    if (bb < w.B) st = *reinterpret_cast<const float2*>(a.stats + ((int64_t)bb * F * w.G + r) * 2);
    t_stats[bs][r] = st;
  }
  for (int i = tid; i < XS_BYTES / 16; i += 256) reinterpret_cast<u32x4_t*>(xs)[i] = u32x4_t{0, 0, 0, 0};
  // frame embedding: requested now, copied into the (still unused) slice-out patch area once the x
  // tile has left LDS; a table too large for that area is read from memory in LN1 instead
  const int pe_n4 = F * (D / 4);
  const bool pe_lds = a.pe != nullptr && pe_n4 * 16 <= PATCH_BYTES;
  constexpr int PE_PER = (PATCH_BYTES / 16 + 255) / 256;
  float4 pev[PE_PER];
#pragma unroll
  for (int i = 0; i < PE_PER; ++i) {
    const int idx = tid + 256 * i;
    pev[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (pe_lds && idx < pe_n4) pev[i] = reinterpret_cast<const float4*>(a.pe)[idx];
  }
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
  float* t_pe = reinterpret_cast<float*>(arena + 4 * SLOT_BYTES);  // [F][D] while the patches are unused
  if (pe_lds) {
#pragma unroll
    for (int i = 0; i < PE_PER; ++i) {
      const int idx = tid + 256 * i;
      if (idx < pe_n4) reinterpret_cast<float4*>(t_pe)[idx] = pev[i];
    }
  }
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
  SI_RING_BARRIER()
#define SI_FRAG(f) fifo[(f) % FIFO]
#define SI_REFILL1(f)                                                                                \
  fifo[(f) % FIFO] = __builtin_bit_cast(bf16x8_t, (f) < FIFO ? slot_c[((f) + FIFO) * kWave + lane]   \
                                                             : slot_n[((f)-FIFO) * kWave + lane])
#define SI_REFILL(f)                                                                                 \
  if constexpr (FIFO % 5 != 0) { SI_REFILL1(f); }                                                    \
  else if ((f) % 5 == 4) { _Pragma("unroll") for (int rj = (f) - 4; rj <= (f); ++rj) { SI_REFILL1(rj); } }
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

  // ---- proj_in; the residual stream is parked in scratch (register image, read back by the same lanes)
  f32x16_t hacc[NB];
  float4* park = reinterpret_cast<float4*>(a.hpark) + ((int64_t)blockIdx.x * 4 + wave) * (NB * 4 * kWave) + lane;
  // The way back: block nb of the parked residual returns through LDS (two 16 KiB landing buffers in
  // the patch area, [wavefront][quad][lane] float4) with the same direct loads as the weight stream,
  // so that its waits are the steps' own closing waits.
  const char* park_s = reinterpret_cast<const char*>(a.hpark) + ((int64_t)blockIdx.x * 4 + pipe_wave) * (NB * 4 * kWave * 16);
  const unsigned park_lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(arena + 4 * SLOT_BYTES) + pipe_wave * (4 * kWave * 16);
  const float4* park_back = reinterpret_cast<const float4*>(arena + 4 * SLOT_BYTES) + wave * (4 * kWave) + lane;
#define SI_PARK_FETCH(nb)                                                                            \
  _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                    \
    const char* sb = park_s + ((nb) * 4 + q) * (kWave * 16);                                         \
    const unsigned l = park_lds + (unsigned)((((nb) % 2) * 16 + q) * (kWave * 16));                  \
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"((unsigned)(lane * 16)), "s"(sb), "s"(l) : "memory"); \
  }
  float4* const hdump = reinterpret_cast<float4*>(a.hpark + ((int64_t)w.B * F * w.Pw + 127) / 128 * 128 * D) + tid;
#define SI_PROJ_IN_BLOCK(nb)                                                                         \
  {                                                                                                  \
    SI_STEP_OPEN();                                                                                  \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) hacc[nb][e] = 0.f;                                \
    _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                                \
      hacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), aop[s], hacc[nb], 0, 0, 0);     \
      SI_REFILL(s);                                                                                  \
      __builtin_amdgcn_sched_barrier(0);                                                             \
    }                                                                                                \
    /* the previous block's 4 park stores are younger than the batch awaited here */                 \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    if ((nb) > 0) Pipe::template wait_step<4>(cur, TOTAL_SUB);                                       \
    else Pipe::template wait_step<0>(cur, TOTAL_SUB);                                                \
    ++cur;                                                                                           \
    __syncthreads();                                                                                 \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                  \
      const float4 bb = *reinterpret_cast<const float4*>(&t_bin[32 * (nb) + 8 * q + 4 * g]);         \
      hacc[nb][4 * q + 0] += bb.x; hacc[nb][4 * q + 1] += bb.y;                                      \
      hacc[nb][4 * q + 2] += bb.z; hacc[nb][4 * q + 3] += bb.w;                                      \
      /* always 4 stores per block (the closing waits count them): idle lanes write to the dump area */ \
      float4* hdst = !SPLIT ? park + ((nb) * 4 + q) * kWave                                          \
                     : row_live ? reinterpret_cast<float4*>(a.hpark) +                                \
                                      h_tile_index<NB>(my_row / 128, nb, q, (int)(my_row % 128) / 32, 32 * g + (int)(my_row % 32)) \
                                : hdump;                                                             \
      *hdst = make_float4(hacc[nb][4 * q + 0], hacc[nb][4 * q + 1], hacc[nb][4 * q + 2], hacc[nb][4 * q + 3]); \
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
    // out = LN1(h0) (+ frame embedding row of this lane's frame); PE4(n) yields columns n .. n+3 of that row
#define SI_LN1_APPLY(PE4)                                                                      \
  _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                            \
  _Pragma("unroll") for (int hf = 0; hf < 2; ++hf) {                                           \
    float v[8];                                                                                \
    _Pragma("unroll") for (int e4 = 0; e4 < 8; e4 += 4) {                                      \
      const int n = 32 * nb + 16 * hf + frag_k(g, e4); /* four consecutive columns */          \
      const float4 gg = *reinterpret_cast<const float4*>(&t_lg[n]);                            \
      const float4 bb = *reinterpret_cast<const float4*>(&t_lb[n]);                            \
      const float4 pp = PE4;                                                                   \
      v[e4 + 0] = (hacc[nb][8 * hf + e4 + 0] - mean) * rstd * gg.x + bb.x + pp.x;              \
      v[e4 + 1] = (hacc[nb][8 * hf + e4 + 1] - mean) * rstd * gg.y + bb.y + pp.y;              \
      v[e4 + 2] = (hacc[nb][8 * hf + e4 + 2] - mean) * rstd * gg.z + bb.z + pp.z;              \
      v[e4 + 3] = (hacc[nb][8 * hf + e4 + 3] - mean) * rstd * gg.w + bb.w + pp.w;              \
    }                                                                                          \
    aop[2 * nb + hf] = to_operand(v);                                                          \
  }
    if (pe_lds) {
      const float* perow = t_pe + my_f * D;
      SI_LN1_APPLY(*reinterpret_cast<const float4*>(perow + n))
    } else if (a.pe) {
      const float* perow = a.pe + (int64_t)my_f * D;
      SI_LN1_APPLY(*reinterpret_cast<const float4*>(perow + n))
    } else {
      SI_LN1_APPLY(make_float4(0.f, 0.f, 0.f, 0.f))
    }
#undef SI_LN1_APPLY
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

  // ---- groups of heads; the attention output is collected as the out-projection's column operands
  u32x4_t oop[SUB];
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
      if (!SPLIT && gi == NG - 1) {  // no more steps until the out-projection: its first two blocks' residual sets out now
        SI_PARK_FETCH(0)
        if (NB > 1) { SI_PARK_FETCH(1) }
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
              if (col >= c0 && col < c1) {
                // heads concatenated: quad q of block blk fills half of the operand of k-step 2*blk + q/2
                const int s2 = 2 * (gi * NBG + blk) + q / 2;
                if (q % 2 == 0) {
                  oop[s2].x = pack_bf16x2(ot[4 * q + 0] * inv, ot[4 * q + 1] * inv);
                  oop[s2].y = pack_bf16x2(ot[4 * q + 2] * inv, ot[4 * q + 3] * inv);
                } else {
                  oop[s2].z = pack_bf16x2(ot[4 * q + 0] * inv, ot[4 * q + 1] * inv);
                  oop[s2].w = pack_bf16x2(ot[4 * q + 2] * inv, ot[4 * q + 3] * inv);
                }
              }
            }
          }
        }
      }
    }
  }
#undef SI_BLOCK_WCOLS
#undef SI_BLOCK_WROWS

  if constexpr (SPLIT) {  // the attention output: oop[s] is the lane's 16 bytes of fragment (token tile, k-step s)
    if (row_live) {
      u32x4_t* of = reinterpret_cast<u32x4_t*>(a.o_rows) + (my_row / 32) * SUB * kWave + 32 * g + (int)(my_row % 32);
#pragma unroll
      for (int s = 0; s < SUB; ++s) of[s * kWave] = oop[s];
    }
    return;
  }
  // ---- h = h0 + o W_o + b_o: NB steps form one 32-column block of o W_o each; the parked residual
  // block (fetched two steps ahead) and the bias are added behind the step
#pragma unroll
  for (int s = 0; s < SUB; ++s) aop[s] = __builtin_bit_cast(bf16x8_t, oop[s]);
#define SI_WO_BLOCK(nb)                                                                             \
  {                                                                                                 \
    SI_STEP_OPEN();                                                                                 \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) hacc[nb][e] = 0.f;                               \
    _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                               \
      hacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), aop[s], hacc[nb], 0, 0, 0);    \
      SI_REFILL(s);                                                                                 \
      __builtin_amdgcn_sched_barrier(0);                                                            \
    }                                                                                               \
    /* block nb's residual must have landed; the fetch of block nb + 1 and the batch of this step */ \
    /* are younger and may stay in flight */                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                              \
    Pipe::wait_step_n(cur, TOTAL_SUB, (nb) + 1 < NB ? 4 : 0);                                       \
    ++cur;                                                                                          \
    __syncthreads();                                                                                \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                 \
      const float4 pk = park_back[(((nb) % 2) * 16 + q) * kWave];                                   \
      hacc[nb][4 * q + 0] += pk.x + t_bo[32 * (nb) + 8 * q + 4 * g + 0];                            \
      hacc[nb][4 * q + 1] += pk.y + t_bo[32 * (nb) + 8 * q + 4 * g + 1];                            \
      hacc[nb][4 * q + 2] += pk.z + t_bo[32 * (nb) + 8 * q + 4 * g + 2];                            \
      hacc[nb][4 * q + 3] += pk.w + t_bo[32 * (nb) + 8 * q + 4 * g + 3];                            \
    }                                                                                               \
    if ((nb) + 2 < NB) { /* this landing buffer is read out: block nb + 2 may overwrite it */       \
      __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0) */                                          \
      SI_PARK_FETCH((nb) + 2)                                                                       \
    }                                                                                               \
  }
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) SI_WO_BLOCK(nb)
#undef SI_WO_BLOCK
#undef SI_PARK_FETCH

  // ---- LN3 over the row (this lane holds half of it, lane ^ 32 the other half); aop becomes its output
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

  // A step issues, per fragment: one MFMA, the fragment's FIFO refill, and one stage of the GEGLU
  // group that rides along (a handful of independent vector-ALU instructions that execute while
  // the matrix pipe works); sched_barrier pins that order.  Stages that do not fit behind the
  // SUB MFMAs run after them.
#define SI_GEGLU_TAIL(GRP, UVC, UGC) \
  _Pragma("unroll") for (int s = SUB; s < kGeluStages; ++s) GRP.stage(s, UVC, UGC, bvp, bgp, gv)
  // W1 sub-chunk into one accumulator block (value or gate rows of a chunk)
#define SI_RUN_W1(ACC, STAGE_STMT)                                                          \
  _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                         \
    if (s == 0) { _Pragma("unroll") for (int e = 0; e < 16; ++e) ACC[e] = 0.f; }            \
    ACC = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), aop[s], ACC, 0, 0, 0);        \
    SI_REFILL(s);                                                                           \
    STAGE_STMT;                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                      \
  }
  // W2 sub-chunk: the chunk's GEGLU output times W2, accumulated into the residual blocks
#define SI_RUN_W2(GOP, STAGE_STMT)                                                                       \
  _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                                      \
    hacc[s / 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), GOP[s % 2], hacc[s / 2], 0, 0, 0); \
    SI_REFILL(s);                                                                                        \
    STAGE_STMT;                                                                                          \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
  }
#define SI_GELU_PACK(GOP)          \
  GOP[0] = to_operand(&gv[0]);     \
  GOP[1] = to_operand(&gv[8])

  // Pipeline slot t: MFMAs of W1(t+1) and W2(t-1), GEGLU of chunk t in three groups of result
  // registers.  Chunk c keeps its W1 results in register set c % 2, its operand in gop set c % 2.
#define SI_SLOT(t, UVC, UGC, UVN, UGN, GOPP, GOPC)                                              \
  {                                                                                                 \
    const float* bvp = t_b1 + 32 * (t) + 4 * g;                                                     \
    const float* bgp = bvp + 4 * D;                                                                 \
    GegluGroup<0, 6> ga;                                                                            \
    GegluGroup<6, 5> gb;                                                                            \
    GegluGroup<11, 5> gc;                                                                           \
    { SI_STEP_OPEN(); SI_RUN_W1(UVN, ga.stage(s, UVC, UGC, bvp, bgp, gv)) SI_GEGLU_TAIL(ga, UVC, UGC); SI_STEP_CLOSE(); } \
    { SI_STEP_OPEN(); SI_RUN_W1(UGN, gb.stage(s, UVC, UGC, bvp, bgp, gv)) SI_GEGLU_TAIL(gb, UVC, UGC); SI_STEP_CLOSE(); } \
    { SI_STEP_OPEN(); SI_RUN_W2(GOPP, gc.stage(s, UVC, UGC, bvp, bgp, gv)) SI_GEGLU_TAIL(gc, UVC, UGC); SI_GELU_PACK(GOPC); SI_STEP_CLOSE(); } \
  }

  f32x16_t uvA, ugA, uvB, ugB;
  bf16x8_t gopA[2], gopB[2];
  float gv[16];
  // prologue: W1(0), then W1(1) with the GEGLU of chunk 0
  { SI_STEP_OPEN(); SI_RUN_W1(uvA, (void)0) SI_STEP_CLOSE(); }
  { SI_STEP_OPEN(); SI_RUN_W1(ugA, (void)0) SI_STEP_CLOSE(); }
  {
    const float* bvp = t_b1 + 4 * g;
    const float* bgp = bvp + 4 * D;
    GegluGroup<0, 8> ga;
    GegluGroup<8, 8> gb;
    { SI_STEP_OPEN(); SI_RUN_W1(uvB, ga.stage(s, uvA, ugA, bvp, bgp, gv)) SI_GEGLU_TAIL(ga, uvA, ugA); SI_STEP_CLOSE(); }
    { SI_STEP_OPEN(); SI_RUN_W1(ugB, gb.stage(s, uvA, ugA, bvp, bgp, gv)) SI_GEGLU_TAIL(gb, uvA, ugA); SI_GELU_PACK(gopA); SI_STEP_CLOSE(); }
  }
  // steady state, two slots per trip (odd chunk in set B, even chunk in set A)
#pragma unroll 1
  for (int t = 1; t <= NC - 2; t += 2) {
    SI_SLOT(t, uvB, ugB, uvA, ugA, gopA, gopB)
    SI_SLOT(t + 1, uvA, ugA, uvB, ugB, gopB, gopA)
  }
  // drain: W2(NC-2) with the GEGLU of the last chunk (set B), then W2(NC-1)
  {
    const float* bvp = t_b1 + 32 * (NC - 1) + 4 * g;
    const float* bgp = bvp + 4 * D;
    GegluGroup<0, 8> ga;
    GegluGroup<8, 8> gb;
#pragma unroll
    for (int s = 0; s < kGeluStages; ++s) ga.stage(s, uvB, ugB, bvp, bgp, gv);
#pragma unroll
    for (int s = 0; s < kGeluStages; ++s) gb.stage(s, uvB, ugB, bvp, bgp, gv);
    SI_GELU_PACK(gopB);
    { SI_STEP_OPEN(); SI_RUN_W2(gopA, (void)0) SI_STEP_CLOSE(); }
    { SI_STEP_OPEN(); SI_RUN_W2(gopB, (void)0) SI_STEP_CLOSE(); }
  }

  // ---- final h (+ b2) as bf16 operands; proj_out one 32-channel block at a time
  bf16x8_t hop[SUB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      float vh[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) vh[e] = hacc[nb][8 * hf + e] + t_b2[32 * nb + 16 * hf + frag_k(g, e)];
      hop[2 * nb + hf] = to_operand(vh);
    }

  // ---- slice-out (see the header comment).  Patch column of this lane's token: frame * NPOS + position.
  const int pcol = my_f * NPOS + wave * TP + my_pp;
  const bool prow = tcol < TP * F;
  const int64_t cs = (int64_t)F * w.P;
  // Pieces of 4 consecutive positions of one (channel row r, frame f) of a block: piece id = tid + 256 i.
  const bool vec_ok = (w.Pw % 4 == 0) && (w.p0 % 4 == 0) && (w.P % 4 == 0);
  const int pieces_per_run = NPOS / 4, pieces = 32 * F * pieces_per_run;  // per block; <= 1024
  int64_t poff[4];  // element offset of the piece in channel 0 of a block
  int pidx[4];      // patch row r and column, packed: r * 1024 + column
  bool plive[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int id = tid + 256 * i;
    const int k = id % pieces_per_run, f = (id / pieces_per_run) % F, r = id / (pieces_per_run * F);
    const int64_t seq = seq_wg + 4 * k;
    plive[i] = vec_ok && id < pieces && seq < nseq;
    const int64_t sq = plive[i] ? seq : 0;
    const int b = (int)sq / w.Pw, pl = (int)sq % w.Pw;
    poff[i] = plive[i] ? (((int64_t)b * w.C + r) * F + f) * w.P + w.p0 + pl : 0;
    pidx[i] = (r < 32 ? r : 0) * 1024 + f * NPOS + 4 * k;
  }
  // x travels two blocks ahead of its use: 4 loads per lane and block, always issued (an idle lane
  // re-reads element 0) so that the closing wait of a step can count them
  uint2 xq[3][4];
  uint2* dummy = reinterpret_cast<uint2*>(a.hpark + (int64_t)blockIdx.x * 128 * D) + tid;  // this workgroup's park area
#define SI_X_LOAD(nbx)                                                                               \
  _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                      \
    xq[(nbx) % 3][i] = *reinterpret_cast<const uint2*>(a.x + poff[i] + (plive[i] ? (int64_t)(32 * (nbx)) * cs : 0))
  SI_X_LOAD(0);
  if (NB > 1) { SI_X_LOAD(1); }

#define SI_PROJ_OUT_BLOCK(nb)                                                                        \
  {                                                                                                  \
    f32x16_t y;                                                                                      \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) y[e] = 0.f;                                       \
    {                                                                                                \
      SI_STEP_OPEN();                                                                                \
      if ((nb) + 2 < NB) { SI_X_LOAD((nb) + 2); }                                                    \
      __builtin_amdgcn_sched_barrier(0);                                                             \
      _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                              \
        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), hop[s], y, 0, 0, 0);                 \
        SI_REFILL(s);                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                           \
      }                                                                                              \
      if (prow) {                                                                                    \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                                \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
          patch[(nb) % 2][8 * q + 4 * g + j][pcol] = y[4 * q + j] + t_bout[32 * (nb) + 8 * q + 4 * g + j]; \
      }                                                                                              \
      /* the barrier publishes the patch; the other patch is free two barriers later */             \
      __builtin_amdgcn_sched_barrier(0);                                                             \
      /* loads and stores younger than the awaited batch stay in flight: x of blocks nb + 1 (nb = 0: */ \
      /* 0 and 1) and nb + 2, and the 4 vector stores of block nb - 1 */                              \
      {                                                                                              \
        const int xe = ((nb) == 0 ? (NB > 1 ? 8 : 4) : ((nb) + 1 < NB ? 4 : 0)) + ((nb) + 2 < NB ? 4 : 0); \
        const int se = (nb) == 0 ? 0 : 4;                                                            \
        Pipe::wait_step_n(cur, TOTAL_SUB, vec_ok ? xe + se : xe);                                    \
      }                                                                                              \
      ++cur;                                                                                         \
      __syncthreads();                                                                               \
    }                                                                                                \
    if (vec_ok) {                                                                                    \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) { /* always 4 stores: idle lanes write to the dead park area */ \
        const float4 yv = *reinterpret_cast<const float4*>(&patch[(nb) % 2][pidx[i] / 1024][pidx[i] % 1024]); \
        const uint2 xr = xq[(nb) % 3][i];                                                            \
        uint2 o;                                                                                     \
        o.x = pack_bf16x2(__uint_as_float(xr.x << 16) + yv.x, __uint_as_float(xr.x & 0xffff0000u) + yv.y); \
        o.y = pack_bf16x2(__uint_as_float(xr.y << 16) + yv.z, __uint_as_float(xr.y & 0xffff0000u) + yv.w); \
        uint2* dst = plive[i] ? reinterpret_cast<uint2*>(a.out + poff[i] + (int64_t)(32 * (nb)) * cs) : dummy + 256 * i; \
        *dst = o;                                                                                    \
      }                                                                                              \
    } else {                                                                                         \
      for (int id = tid; id < 32 * F * NPOS; id += 256) {                                            \
        const int j = id % NPOS, f = (id / NPOS) % F, r = id / (NPOS * F);                           \
        const int64_t seq = seq_wg + j;                                                              \
        if (seq < nseq) {                                                                            \
          const int64_t off = (((int64_t)((int)seq / w.Pw) * w.C + 32 * (nb) + r) * F + f) * w.P + w.p0 + ((int)seq % w.Pw); \
          a.out[off].v = float_to_bf16_bits(bf16_bits_to_float(a.x[off].v) + patch[(nb) % 2][r][f * NPOS + j]); \
        }                                                                                            \
      }                                                                                              \
    }                                                                                                \
  }
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) SI_PROJ_OUT_BLOCK(nb)
#undef SI_PROJ_OUT_BLOCK
#undef SI_X_LOAD
#undef SI_SLOT
#undef SI_GELU_PACK
#undef SI_RUN_W2
#undef SI_RUN_W1
#undef SI_GEGLU_TAIL
#undef SI_REFILL
#undef SI_REFILL1
#undef SI_FRAG
#undef SI_STEP_CLOSE
#undef SI_STEP_OPEN
}

}  // namespace si
