// Register-resident fused kernels for blocks whose inner width D = 32*NB fits a
// wavefront's register file (D <= 320, C == D, bf16 storage).
//
// Idea.  In v_mfma_f32_32x32x16_bf16 the row operand and the column operand
// have the same register shape: lane l supplies 8 k-values (slot g = l/32) of
// row / column l%32.  The result gives lane l column l%32 and, in register
// quad q, rows 8q + 4g + {0..3}.  If tokens are the COLUMNS, a lane's 16 result
// registers of a 32-row block, converted to bf16, are exactly the column
// operand of the next contraction for the two 16-wide k-steps of that block --
// provided the weight fragments of the next contraction list their k-values in
// the order k(g, e) = 16s + (e < 4 ? 4g + e : 8 + 4g + e - 4).  The weights are
// re-laid-out once per call into that order ("fragment stream": 1 KiB per
// (32-row block, k-step), in exactly the order the kernel consumes them).
//
// So one wavefront carries 32 tokens through a whole operator chain without
// its activations ever leaving registers; the only LDS traffic is the weight
// stream, loaded once per workgroup (4 wavefronts x 32 tokens) into a ring of
// sub-chunks of 2*NB fragments and read by all four wavefronts.
//
//   ffn_half_kernel   h (fp32 rows) -> LN3 -> W1 -> GEGLU -> W2 (+h) -> W_out
//                     -> + x -> out window.  The 8D-wide FFN intermediate and
//                     the final h exist only in registers.  The FFN runs as a
//                     three-stage software pipeline over 32-column chunks so
//                     that the GELU arithmetic of chunk t issues between the
//                     MFMAs of chunks t+1 (W1) and t-1 (W2).
#pragma once
#include <type_traits>

#include "si_common.h"
#include "k_norm.h"

namespace si {

// Compile-time loop: f(std::integral_constant<int, I>) for I in [0, N).
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// Logical k offset inside a 16-wide k-step of hardware slot (g, e).
__host__ __device__ __forceinline__ int frag_k(int g, int e) { return e < 4 ? 4 * g + e : 8 + 4 * g + (e - 4); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

// 8 consecutive result registers (two quads) -> column operand of one k-step.
__device__ __forceinline__ bf16x8_t to_operand(const float* v) {
  uint4 u;
  u.x = pack_bf16x2(v[0], v[1]);
  u.y = pack_bf16x2(v[2], v[3]);
  u.z = pack_bf16x2(v[4], v[5]);
  u.w = pack_bf16x2(v[6], v[7]);
  return __builtin_bit_cast(bf16x8_t, u);
}

// GELU(x) = x * Phi(x), Phi(x) = 0.5 (1 + erf(x / sqrt 2)).  Phi(x) - 0.5 is evaluated as an odd
// polynomial xc * R(xc^2), xc = clamp(x, -4.2, 4.2), degree 8 in xc^2 (minimax fit of
// erf(x / sqrt 2) / x on [0, 4.2], |erf error| <= 2.2e-5 everywhere, coefficients pre-halved).
// No transcendental instructions: the FFN's GELUs share the issue port with the MFMAs.
// (kGeluClamp, kGeluDeg, kGeluC: si_common.h)

// GEGLU of G result registers [E0, E0+G) of one chunk, cut into stages of G independent
// vector-ALU instructions each, so that one stage can be issued behind every MFMA.
//   value = UV[e] + bv[off(e)], gate = UG[e] + bg[off(e)], gv[e] = value * gate * Phi(gate)
// off(e): column of result register e relative to the lane's first column (see frag_k).
__host__ __device__ constexpr int reg_col(int e) { return 16 * (e / 8) + ((e % 8) < 4 ? (e % 8) : (e % 8) + 4); }
constexpr int kGeluStages = kGeluDeg + 11;

// Stage 0 only issues the LDS reads of the group's biases; they are consumed three stages (three
// MFMAs) later, so no stage waits for a read issued just before it.
template <int E0, int G>
struct GegluGroup {
  float x[G], v[G], xc[G], t[G], p[G], bgr[G], bvr[G];
  __device__ __forceinline__ void stage(int s, const f32x16_t& UV, const f32x16_t& UG, const float* bv, const float* bg,
                                        float* gv) {
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const int e = E0 + i;
      if (s == 0) bgr[i] = bg[reg_col(e)];
      else if (s == 1) bvr[i] = bv[reg_col(e)];
      else if (s == 2) x[i] = UG[e];
      else if (s == 3) v[i] = UV[e];
      else if (s == 4) x[i] += bgr[i];
      else if (s == 5) v[i] += bvr[i];
      else if (s == 6) xc[i] = __builtin_amdgcn_fmed3f(x[i], -kGeluClamp, kGeluClamp);
      else if (s == 7) t[i] = xc[i] * xc[i];
      else if (s == 8) p[i] = fmaf(kGeluC[kGeluDeg], t[i], kGeluC[kGeluDeg - 1]);
      else if (s >= 9 && s < 8 + kGeluDeg) p[i] = fmaf(p[i], t[i], kGeluC[kGeluDeg + 7 - s]);
      else if (s == 8 + kGeluDeg) p[i] = fmaf(p[i], xc[i], 0.5f);  // Phi(gate)
      else if (s == 9 + kGeluDeg) x[i] = x[i] * v[i];
      else if (s == 10 + kGeluDeg) gv[e] = x[i] * p[i];
    }
  }
};

// ----------------------------------------------------------------------------- weight stream layout

// Placement of the fragment stream in memory.  Every workgroup reads the same
// fragments at about the same time, so the fragments of one sub-chunk are kept
// out of a single L2 channel: fragment f of sub-chunk i lives at 16-byte index
// f * pitch + i * 64 (+ lane), pitch an odd number of KiB (in 16-byte units)
// congruent to 5 mod 16.
__host__ __device__ inline int64_t stream_pitch_u4(int total_sub) {
  int kib = total_sub;
  while (kib % 16 != 5) ++kib;
  return (int64_t)kib * 64;
}
__host__ __device__ inline int64_t stream_bytes(int total_sub, int sub) { return stream_pitch_u4(total_sub) * 16 * sub; }

// Fragment stream, in consumption order.  A sub-chunk is 2*NB fragments (fragment = 64 lanes x
// 8 bf16).  Block sub-chunks: one 32-column block of a row-major [D, ld] matrix, k-steps 0..2NB-1
// over its D rows (proj_in, q/k/v, attention out-projection, proj_out).  FFN sub-chunks, with
// NC = 4*NB chunks of 32 inner columns:
//   V(c): W1 value rows 32c..32c+31, k-steps 0..2NB-1      G(c): the gate rows likewise
//   W2(c): for nb in [0, NB): k-steps (inner 32c..32c+15), (32c+16..32c+31)
// order: V0 G0 V1 G1 | for t in 1..NC-2: V(t+1) G(t+1) W2(t-1) | W2(NC-2) W2(NC-1)
// One thread per (fragment, lane).  Sources are row-major [in, out].
struct BlockDesc {
  const bf16* src;
  int ld, col0;
  int f16;  // store the values as fp16 (operands of an fp16 contraction)
};

// Whole fragment stream in one launch: n_pre block sub-chunks, the FFN's 12*NB sub-chunks, n_post
// block sub-chunks, and -- in further workgroups -- the
// sinusoidal frame table PE[f, 2i] = sin(f / 10000^(2i/D)), PE[f, 2i+1] = cos(same) when pe != NULL.
struct StreamDesc {
  BlockDesc b[64];  // pre blocks first, then post blocks
  int n_pre, n_post;
  int n_ffn;  // 12 * NB, or 0 for a stream of blocks only
  const bf16 *w1, *w2;
  float* pe;
  int F;
  int extra_sub;  // sub-chunks that another kernel appends behind these (they share the stream's pitch)
};
template <int NB>
__global__ __launch_bounds__(256) void pack_stream_kernel(StreamDesc sd, u32x4_t* __restrict__ dst) {
  constexpr int D = 32 * NB, SUB = 2 * NB, NC = 4 * NB;
  const int total_sub = sd.n_pre + sd.n_ffn + sd.n_post;
  const int frag_wgs = (total_sub * SUB + 3) / 4;
  if ((int)blockIdx.x >= frag_wgs) {  // frame table
    const int idx = ((int)blockIdx.x - frag_wgs) * 256 + threadIdx.x;
    if (sd.pe && idx < sd.F * D) {
      const int f = idx / D, i = idx % D;
      const int even = i - (i & 1);
      const double angle = (double)f / pow(10000.0, (double)even / (double)D);
      sd.pe[idx] = (float)((i & 1) ? cos(angle) : sin(angle));
    }
    return;
  }
  const int fidx = blockIdx.x * 4 + threadIdx.x / kWave;
  if (fidx >= total_sub * SUB) return;
  const int lane = threadIdx.x % kWave, r = lane % 32, g = lane / 32;
  const int sub = fidx / SUB, idx = fidx % SUB;
  const bf16* src;
  int ld, n, k0, f16 = 0;
  if (sub < sd.n_pre || sub >= sd.n_pre + sd.n_ffn) {
    const BlockDesc d = sd.b[sub < sd.n_pre ? sub : sub - sd.n_ffn];
    src = d.src; ld = d.ld; n = d.col0 + r; k0 = 16 * idx; f16 = d.f16;
  } else {
    const int fs = sub - sd.n_pre;
    int kind, c;  // kind 0: V, 1: G, 2: W2
    if (fs < 4) {
      kind = fs % 2; c = fs / 2;
    } else if (fs < 4 + 3 * (NC - 2)) {
      const int rr = fs - 4, t = 1 + rr / 3, k = rr % 3;
      kind = k; c = k == 2 ? t - 1 : t + 1;
    } else {
      kind = 2; c = NC - 2 + (fs - (4 + 3 * (NC - 2)));
    }
    if (kind < 2) {
      src = sd.w1; ld = 8 * D; n = (kind ? 4 * D : 0) + 32 * c + r; k0 = 16 * idx;
    } else {
      src = sd.w2; ld = D; n = 32 * (idx / 2) + r; k0 = 32 * c + 16 * (idx % 2);
    }
  }
  unsigned short e[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    e[i] = src[(int64_t)(k0 + frag_k(g, i)) * ld + n].v;
    if (f16) e[i] = __builtin_bit_cast(unsigned short, (_Float16)__builtin_amdgcn_fmed3f(bf16_bits_to_float(e[i]), -65504.f, 65504.f));
  }
  u32x4_t o;
  o.x = e[0] | ((unsigned)e[1] << 16);
  o.y = e[2] | ((unsigned)e[3] << 16);
  o.z = e[4] | ((unsigned)e[5] << 16);
  o.w = e[6] | ((unsigned)e[7] << 16);
  dst[idx * stream_pitch_u4(total_sub + sd.extra_sub) + (int64_t)sub * kWave + lane] = o;
}

// ----------------------------------------------------------------------------- weight stream pipeline

// The workgroup moves the fragment stream through a ring of kRingSlots LDS slots of SUB fragments
// with direct global-to-LDS loads (global_load_lds_dwordx4: lane i of a wavefront deposits its 16
// bytes at LDS address M0 + 16 i, i.e. one fragment per instruction, no staging registers).  At the
// start of step i the loads of sub-chunk i+3 are issued into slot (i+3) % 4 -- the slot read in
// step i-1; the MFMAs of sub-chunk i read slot i % 4 and, through the register FIFO's refills,
// slot (i+1) % 4.  Before the barrier that closes step i every wavefront waits until at most its
// newest batch of loads is outstanding (loads return in issue order), so sub-chunk i+2 is in LDS
// for everybody two steps before it becomes the FIFO's refill source.
#ifndef SI_RING_SLOTS
#define SI_RING_SLOTS 4
#endif
constexpr int kRingSlots = SI_RING_SLOTS;
// The barrier that closes a step of the ring.  What it orders is (1) every wavefront's own
// global->LDS loads of sub-chunk cur + 2, awaited through vmcnt just before, and (2) the reads of
// the slot that the loads issued right after it overwrite -- the slot of the step before, whose
// last reads were consumed (hence complete) ten MFMAs ago.  LDS reads issued in the step that
// closes target slots that stay untouched for two more steps, so they need not have returned: a
// bare s_barrier, without the wait for all LDS traffic that __syncthreads() adds.
#define SI_RING_BARRIER() __builtin_amdgcn_s_barrier()
static_assert(kRingSlots >= 4 && kRingSlots <= 6, "ring depth");
template <int SUB>
struct WeightPipe {
  static constexpr int PER_THREAD = SUB * kWave / 256;  // loads per lane per sub-chunk
  // s_waitcnt immediate (gfx9 encoding): vmcnt <= n, other counters unconstrained
  static constexpr int wait_imm(int n) { return (n & 0xF) | 0x70 | 0xF00 | ((n >> 4) << 14); }
  // Closing wait of step `cur`: sub-chunk cur + 2 must have landed.  Younger batches (up to
  // kRingSlots - 3 of them, fewer at the stream's tail) and EXTRA loads issued after them may stay
  // in flight.
  template <int EXTRA = 0>
  static __device__ __forceinline__ void wait_step(int cur, int total) {
    int n = total - 3 - cur;
    n = n < kRingSlots - 3 ? n : kRingSlots - 3;
    if (n <= 0) __builtin_amdgcn_s_waitcnt(wait_imm(EXTRA));
    else if (n == 1) __builtin_amdgcn_s_waitcnt(wait_imm(PER_THREAD + EXTRA));
    else if (n == 2) __builtin_amdgcn_s_waitcnt(wait_imm(2 * PER_THREAD + EXTRA));
    else __builtin_amdgcn_s_waitcnt(wait_imm(3 * PER_THREAD + EXTRA));
  }
  // same with a run-time count (rounded down to a multiple of 4, at most 12; constant after unrolling)
  static __device__ __forceinline__ void wait_step_n(int cur, int total, int extra) {
    if (extra >= 12) wait_step<12>(cur, total);
    else if (extra >= 8) wait_step<8>(cur, total);
    else if (extra >= 4) wait_step<4>(cur, total);
    else wait_step<0>(cur, total);
  }
  // Loads of sub-chunk `sub`.  voff = pipe_voff(lane, wave, pitch): the lane's byte offset inside a
  // sub-chunk's first fragment row of its wavefront; wave_s: the wavefront index as a scalar.  The
  // address is formed as scalar base + 32-bit lane offset, so a step's loads cost scalar
  // instructions only.
  static __device__ __forceinline__ unsigned pipe_voff(int lane, int wave, int64_t pitch) {
    return (unsigned)((lane + (int64_t)wave * pitch) * 16);
  }
  static __device__ __forceinline__ void issue(const u32x4_t* stream, u32x4_t* ring0, int sub, int total, int64_t pitch,
                                               unsigned voff, int wave_s) {
    if (sub < total) issue_at(stream, ring0, sub, sub, pitch, voff, wave_s);
  }
  // Sub-chunk `src_sub` of the stream into the ring slot of step `step` (the two differ where a
  // kernel splices sub-chunks from elsewhere in the stream into its sequence of steps).
  static __device__ __forceinline__ void issue_at(const u32x4_t* stream, u32x4_t* ring0, int src_sub, int step, int64_t pitch,
                                                  unsigned voff, int wave_s) {
    const char* sbase = reinterpret_cast<const char*>(stream) + (int64_t)src_sub * (kWave * 16);
    // LDS byte address of this wavefront's first fragment in the slot, wave-uniform (goes to M0)
    const unsigned dst = (unsigned)(size_t)(__attribute__((address_space(3))) void*)ring0 +
                         (unsigned)((step % kRingSlots) * (SUB * kWave * 16) + wave_s * (kWave * 16));
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const char* sb = sbase + (int64_t)(4 * i) * pitch * 16;
      const unsigned l = dst + (unsigned)(4 * i * kWave * 16);
      // Issued as assembly so that the compiler's wait-count pass does not place a full vector-memory
      // wait in front of every later LDS read; completion is awaited explicitly when a step closes.
      // M0 is reserved by the compiler and used by nothing else in these kernels.
      asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(sb), "s"(l) : "memory");
    }
  }
};

// ----------------------------------------------------------------------------- FFN half

struct FfnHalfArgs {
  const float* h;         // [M, D] residual stream before the last attention output projection
  const bf16* o;          // [M, D] attention output (heads concatenated); h += o W_o + b_o comes first
  int64_t M;
  const u32x4_t* stream;  // fragment stream: W_o blocks, FFN, W_out blocks
  const bf16 *b_o, *ln_g, *ln_b, *b1, *b2, *b_out;
  float ln_eps;
  const bf16* x;
  bf16* out;
  Window win;
  // CROSS only (spatial blocks, heads of 64): `o` / b_o belong to the self-attention; then LN2, the
  // query projection, attention over the context tokens and its out-projection (b_o2) run here too.
  const bf16 *ln2_g, *ln2_b, *b_o2;
  int64_t pitch;          // the stream's pitch in 16-byte units (it also carries the context fragments)
  int ctx_sub0;           // first context sub-chunk of batch entry 0; kCrossSub per batch entry
  int Mc;                 // context tokens (<= 32 * kCrossTiles)
  int tokens_per_batch;   // a multiple of 128: a workgroup's tokens share one context
  float qscale;           // softmax scale * log2(e)
  const bf16* o2;         // with h_tiled, or NULL: the attention ran in two key halves; o / o2 hold each half's
  const float2* ml;       // output and ml[(half * heads + head) * tiles32 + tile][lane] its (reference maximum in
  int64_t tiles32;        // base-2 exponent units, row sum); the halves are merged as the operands are loaded
  int h_tiled;            // h is in workgroup-tile order (h_tile_index) and o holds the attention output as
                          // fragments ([32-token tile][k-step][lane]), as the kernels in front of this one leave them
};

// Residual stream between two register-resident kernels of the same tiling (workgroup = 128 tokens,
// wavefront = 32, lane = (token r, half g), result quad q of 32-channel block nb): index of the
// lane's float4 -- 64 lanes of a wavefront are 1 KiB contiguous.
template <int NB>
__host__ __device__ __forceinline__ int64_t h_tile_index(int64_t tile, int nb, int q, int wave, int lane) {
  return ((((int64_t)tile * NB + nb) * 4 + q) * 4 + wave) * kWave + lane;
}

// Attention over the context inside the FFN-half kernel: up to 3 tiles of 32 keys, heads of 64
// channels.  Per head 24 MFMAs, in this order (= the order of the head's fragments in the stream):
//   j < 12:  S^T[kt] += K[kt, ks] q[ks]         ks = j / 3 (16 head channels), kt = j % 3 (32 keys)
//   j >= 12: O^T[cb] += V^T[cb, kk] P^T[kk]     kk = (j - 12) / 2 (16 keys), cb = (j - 12) % 2 (32 channels)
// so a batch entry's context is 24 * heads fragments = kCrossSub sub-chunks of SUB at 5 heads.
constexpr int kCrossTiles = 3, kCrossOps = 8 * kCrossTiles;

// Context keys / values [B*Mc, 2D] (keys in columns [0, D), values in [D, 2D)) -> the fragments
// above, appended to a fragment stream as sub-chunks sub0 + (NH * kCrossOps / SUB) * b + ...
// Keys past Mc are zero (their scores are masked, their probabilities zero).  One wavefront per fragment.
template <int NB>
__global__ __launch_bounds__(256) void pack_ctx_stream_kernel(const bf16* __restrict__ kv, int B, int Mc, u32x4_t* __restrict__ dst,
                                                              int64_t pitch, int sub0) {
  constexpr int D = 32 * NB, SUB = 2 * NB, NH = D / 64, PERB = NH * kCrossOps;
  static_assert(PERB % SUB == 0, "whole sub-chunks per batch entry");
  const int fidx = blockIdx.x * 4 + threadIdx.x / kWave;
  if (fidx >= B * PERB) return;
  const int lane = threadIdx.x % kWave, r = lane % 32, g = lane / 32;
  const int b = fidx / PERB, i = fidx % PERB, hd = i / kCrossOps, j = i % kCrossOps;
  unsigned short e[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    int key, col;
    if (j < 4 * kCrossTiles) {
      key = 32 * (j % kCrossTiles) + r;
      col = 64 * hd + 16 * (j / kCrossTiles) + frag_k(g, t);
    } else {
      const int jj = j - 4 * kCrossTiles;
      key = 16 * (jj / 2) + frag_k(g, t);
      col = D + 64 * hd + 32 * (jj % 2) + r;
    }
    e[t] = key < Mc ? kv[((int64_t)b * Mc + key) * (2 * D) + col].v : (unsigned short)0;
  }
  u32x4_t o;
  o.x = e[0] | ((unsigned)e[1] << 16);
  o.y = e[2] | ((unsigned)e[3] << 16);
  o.z = e[4] | ((unsigned)e[5] << 16);
  o.w = e[6] | ((unsigned)e[7] << 16);
  const int sub = sub0 + (PERB / SUB) * b + i / SUB;
  dst[(i % SUB) * pitch + (int64_t)sub * kWave + lane] = o;
}

template <int NB, bool CROSS = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void ffn_half_kernel(FfnHalfArgs a) {
  constexpr int D = 32 * NB, SUB = 2 * NB, NC = 4 * NB;  // SUB fragments per sub-chunk (= k-steps over D)
  constexpr int NSLOT = kRingSlots, FIFO = NB;
  // CROSS: W_o, W_q2 blocks | the batch entry's context fragments | W_o2 blocks, FFN, W_out blocks
  constexpr int kCrossSub = CROSS ? (D / 64) * kCrossOps / SUB : 0, kSplice = 2 * NB;
  constexpr int TOTAL_SUB = (CROSS ? 2 * NB : 0) + kCrossSub + NB + 3 * NC + NB;  // steps
  static_assert(NB % 2 == 0, "NB must be even");  // whole fragments per wavefront per sub-chunk
  static_assert(!CROSS || ((D / 64) * kCrossOps) % SUB == 0, "context fragments fill whole sub-chunks");
  __shared__ u32x4_t ring[NSLOT][SUB * kWave];
  __shared__ float t_g[D], t_b[D], t_b2[D], t_bout[D], t_bo[D], t_b1[8 * D];
  __shared__ float t_g2[CROSS ? D : 1], t_bl2[CROSS ? D : 1], t_bo2[CROSS ? D : 1];
  __shared__ __attribute__((aligned(16))) float stage[4][32][36];  // slice-out transpose, one patch per wavefront

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int tcol = lane % 32, g = lane / 32;
  const int64_t m = (int64_t)blockIdx.x * 128 + wave * 32 + tcol;
  const bool live = m < a.M;

  // ---- residual rows into result-layout registers: hacc[nb][4q + j] = h[m][32nb + 8q + 4g + j]
  f32x16_t hacc[NB];
  {
    const float* hrow = a.h + (live ? m : 0) * D;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.h_tiled) {
          if (live) v = reinterpret_cast<const float4*>(a.h)[h_tile_index<NB>(blockIdx.x, nb, q, wave, lane)];
        } else if (live) v = *reinterpret_cast<const float4*>(hrow + 32 * nb + 8 * q + 4 * g);
        hacc[nb][4 * q + 0] = v.x; hacc[nb][4 * q + 1] = v.y; hacc[nb][4 * q + 2] = v.z; hacc[nb][4 * q + 3] = v.w;
      }
  }
  // attention output rows as column operands: k-step s holds o[m][16s + {4g..4g+3, 8+4g..8+4g+3}]
  bf16x8_t aop[SUB];
  {
    const bf16* orow = a.o + (live ? m : 0) * D;
    // two key halves: softmax weights of the halves per head, w = l 2^(m - max m) / sum of the same
    float w0[CROSS ? NB / 2 : 1], w1[CROSS ? NB / 2 : 1];
    const int64_t t32 = (int64_t)blockIdx.x * 4 + wave;
    if (CROSS && a.h_tiled && a.o2) {
#pragma unroll
      for (int hd = 0; hd < NB / 2; ++hd) {
        const float2 p0 = a.ml[((int64_t)hd * a.tiles32 + t32) * kWave + lane];
        const float2 p1 = a.ml[((int64_t)(NB / 2 + hd) * a.tiles32 + t32) * kWave + lane];
        const float mx = fmaxf(p0.x, p1.x);
        const float a0 = p0.y * __builtin_amdgcn_exp2f(p0.x - mx), a1 = p1.y * __builtin_amdgcn_exp2f(p1.x - mx);
        const float inv = 1.0f / (a0 + a1);
        w0[hd] = a0 * inv;
        w1[hd] = a1 * inv;
      }
    }
#pragma unroll
    for (int s2 = 0; s2 < SUB; ++s2) {
      if (a.h_tiled) {  // fragments as the attention kernel leaves them: [32-token tile][k-step][lane]
        const u32x4_t f0 = live ? reinterpret_cast<const u32x4_t*>(a.o)[(t32 * SUB + s2) * kWave + lane] : u32x4_t{0, 0, 0, 0};
        if (CROSS && a.o2) {
          const u32x4_t f1 = reinterpret_cast<const u32x4_t*>(a.o2)[(t32 * SUB + s2) * kWave + lane];
          const float u0 = w0[CROSS ? s2 / 4 : 0], u1 = w1[CROSS ? s2 / 4 : 0];
          const unsigned x0[4] = {f0.x, f0.y, f0.z, f0.w}, x1[4] = {f1.x, f1.y, f1.z, f1.w};
          float v[8];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v[2 * i] = u0 * __uint_as_float(x0[i] << 16) + u1 * __uint_as_float(x1[i] << 16);
            v[2 * i + 1] = u0 * __uint_as_float(x0[i] & 0xffff0000u) + u1 * __uint_as_float(x1[i] & 0xffff0000u);
          }
          aop[s2] = to_operand(v);
        } else {
          aop[s2] = __builtin_bit_cast(bf16x8_t, f0);
        }
        continue;
      }
      uint2 lo = make_uint2(0, 0), hi = make_uint2(0, 0);
      if (live) {
        lo = *reinterpret_cast<const uint2*>(orow + 16 * s2 + 4 * g);
        hi = *reinterpret_cast<const uint2*>(orow + 16 * s2 + 8 + 4 * g);
      }
      u32x4_t u;
      u.x = lo.x; u.y = lo.y; u.z = hi.x; u.w = hi.y;
      aop[s2] = __builtin_bit_cast(bf16x8_t, u);
    }
  }
  for (int i = tid; i < D; i += 256) {
    t_g[i] = param_or(a.ln_g, i, 1.f);
    t_b[i] = param_or(a.ln_b, i, 0.f);
    t_b2[i] = param_or(a.b2, i, 0.f);
    t_bout[i] = param_or(a.b_out, i, 0.f);
    t_bo[i] = param_or(a.b_o, i, 0.f);
    if constexpr (CROSS) {
      t_g2[i] = param_or(a.ln2_g, i, 1.f);
      t_bl2[i] = param_or(a.ln2_b, i, 0.f);
      t_bo2[i] = param_or(a.b_o2, i, 0.f);
    }
  }
  for (int i = tid; i < 8 * D; i += 256) t_b1[i] = param_or(a.b1, i, 0.f);

  // ---- weight stream: the first three sub-chunks go straight into the ring
  using Pipe = WeightPipe<SUB>;
  const int64_t pitch = CROSS ? a.pitch : stream_pitch_u4(TOTAL_SUB);
  const unsigned pipe_voff = Pipe::pipe_voff(lane, wave, pitch);
  const int pipe_wave = __builtin_amdgcn_readfirstlane(wave);
  // the workgroup's context sub-chunks (all of its tokens belong to one batch entry)
  const int ctx_sub = CROSS ? a.ctx_sub0 + kCrossSub * ((int)(blockIdx.x * 128) / a.tokens_per_batch) : 0;
  // loads of step G: the stream's sub-chunk G, except that the context sub-chunks are spliced in
  // behind the first kSplice steps
  auto issue_step = [&](int G) {
    if (G >= TOTAL_SUB) return;
    int src = G;
    if constexpr (CROSS) {
      if (G >= kSplice) src = G < kSplice + kCrossSub ? ctx_sub + (G - kSplice) : G - kCrossSub;
    }
    Pipe::issue_at(a.stream, ring[0], src, G, pitch, pipe_voff, pipe_wave);
  };
  int cur = 0;  // sub-chunk being consumed; loads run at cur + 3
#pragma unroll
  for (int i = 0; i < NSLOT - 1; ++i) issue_step(i);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): also the residual / attention rows loaded above
  __syncthreads();  // tables and the first three sub-chunks are in LDS

  // ---- fragment FIFO: the first FIFO fragments of sub-chunk 0
  bf16x8_t fifo[FIFO];
#pragma unroll
  for (int i = 0; i < FIFO; ++i) fifo[i] = __builtin_bit_cast(bf16x8_t, ring[0][i * kWave + lane]);

  // One pipeline step around the MFMAs of sub-chunk `cur` (see WeightPipe).
#define SI_STEP_OPEN()                                                           \
  __builtin_amdgcn_sched_barrier(0);                                             \
  issue_step(cur + NSLOT - 1);                                                   \
  const u32x4_t* slot_c = ring[cur % NSLOT];                                     \
  const u32x4_t* slot_n = ring[(cur + 1) % NSLOT];                               \
  (void)slot_c; (void)slot_n
#define SI_STEP_CLOSE()                                                          \
  __builtin_amdgcn_sched_barrier(0);                                             \
  Pipe::template wait_step<0>(cur, TOTAL_SUB);                                   \
  ++cur;                                                                         \
  SI_RING_BARRIER()
  // as above when EXTRA (0 or 2) further loads were issued after this step's weight loads
#define SI_STEP_CLOSE_EXTRA(EXTRA)                                               \
  __builtin_amdgcn_sched_barrier(0);                                             \
  if ((EXTRA) == 2) Pipe::template wait_step<2>(cur, TOTAL_SUB);                 \
  else Pipe::template wait_step<0>(cur, TOTAL_SUB);                              \
  ++cur;                                                                         \
  SI_RING_BARRIER()
  // fragment f of the current sub-chunk, and its replacement FIFO fragments further down the stream
#define SI_FRAG(f) fifo[(f) % FIFO]
#define SI_REFILL(f)                                                                                 \
  fifo[(f) % FIFO] = __builtin_bit_cast(bf16x8_t, (f) < FIFO ? slot_c[((f) + FIFO) * kWave + lane]   \
                                                             : slot_n[((f)-FIFO) * kWave + lane])
  // ---- h += o W + b: NB steps, one 32-column block of the residual each (OPS: the k-steps of o as
  // column operands, TB: the bias table)
#define SI_WO_BLOCK(nb, OPS, TB)                                                                 \
  {                                                                                                 \
    SI_STEP_OPEN();                                                                                \
    _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                               \
      hacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), OPS[s], hacc[nb], 0, 0, 0);    \
      SI_REFILL(s);                                                                                 \
      __builtin_amdgcn_sched_barrier(0);                                                            \
    }                                                                                               \
    SI_STEP_CLOSE();                                                                               \
    _Pragma("unroll") for (int q = 0; q < 4; ++q)                                                   \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) hacc[nb][4 * q + j] += TB[32 * (nb) + 8 * q + 4 * g + j]; \
  }
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) SI_WO_BLOCK(nb, aop, t_bo)

  // LayerNorm over the row (this lane holds half of it, lane ^ 32 the other half); aop becomes its output
  auto layer_norm_row = [&](const float* tg, const float* tb) {
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
          v[e] = (hacc[nb][8 * hf + e] - mean) * rstd * tg[n] + tb[n];
        }
        aop[2 * nb + hf] = to_operand(v);
      }
  };

  if constexpr (CROSS) {
    // ---- LN2, then q = LN2(h) W_q2 * scale * log2(e): block nb of the result is k-steps 2nb, 2nb + 1
    // of the score contraction's column operand (head nb / 2)
    layer_norm_row(t_g2, t_bl2);
    bf16x8_t xop[SUB];  // the queries; head by head replaced by the attention output
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      f32x16_t qa;
#pragma unroll
      for (int e = 0; e < 16; ++e) qa[e] = 0.f;
      {
        SI_STEP_OPEN();
#pragma unroll
        for (int s = 0; s < SUB; ++s) {
          qa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), aop[s], qa, 0, 0, 0);
          SI_REFILL(s);
          __builtin_amdgcn_sched_barrier(0);
        }
        SI_STEP_CLOSE();
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = qa[8 * hf + e] * a.qscale;
        xop[2 * nb + hf] = to_operand(v);
      }
    }
    // ---- attention over the context, head by head (see kCrossOps); scores, probabilities and the
    // output stay in registers: keys are the rows of S^T, so a lane holds 16 of a tile's 32 keys of
    // its token and lane ^ 32 the other 16
    f32x16_t sc[kCrossTiles], oc[2];
    bf16x8_t pk[2 * kCrossTiles];
    float inv_l = 0.f;
    static_for<kCrossSub>([&](auto C6) {
      constexpr int c6 = decltype(C6)::value;
      SI_STEP_OPEN();
      static_for<SUB>([&](auto S20) {
        constexpr int s = decltype(S20)::value, i = SUB * c6 + s, hd = i / kCrossOps, j = i % kCrossOps;
        if constexpr (j < 4 * kCrossTiles) {
          constexpr int ks = j / kCrossTiles, kt = j % kCrossTiles;
          if constexpr (ks == 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[kt][e] = 0.f;
          }
          sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), xop[4 * hd + ks], sc[kt], 0, 0, 0);
        } else {
          constexpr int jj = j - 4 * kCrossTiles, kk = jj / 2, cb = jj % 2;
          if constexpr (jj == 0) {  // softmax over the keys (register 4q + j of tile kt: key 32kt + 8q + 4g + j)
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < kCrossTiles; ++kt)
#pragma unroll
              for (int e = 0; e < 16; ++e) {
                if (32 * kt + 8 * (e / 4) + 4 * g + (e % 4) >= a.Mc) sc[kt][e] = -INFINITY;
                mx = fmaxf(mx, sc[kt][e]);
              }
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));  // key 0 exists: finite
            float l = 0.f;
#pragma unroll
            for (int kt = 0; kt < kCrossTiles; ++kt) {
#pragma unroll
              for (int e = 0; e < 16; ++e) {
                sc[kt][e] = __builtin_amdgcn_exp2f(sc[kt][e] - mx);
                l += sc[kt][e];
              }
#pragma unroll
              for (int hf = 0; hf < 2; ++hf) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = sc[kt][8 * hf + e];
                pk[2 * kt + hf] = to_operand(v);
              }
            }
            l += __shfl_xor(l, 32, kWave);
            inv_l = 1.0f / l;
          }
          if constexpr (kk == 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) oc[cb][e] = 0.f;
          }
          oc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), pk[kk], oc[cb], 0, 0, 0);
          if constexpr (jj == 4 * kCrossTiles - 1) {  // the head's output replaces its queries
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
              for (int hf = 0; hf < 2; ++hf) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = oc[b2][8 * hf + e] * inv_l;
                xop[4 * hd + 2 * b2 + hf] = to_operand(v);
              }
          }
        }
        SI_REFILL(s);
        __builtin_amdgcn_sched_barrier(0);
      });
      SI_STEP_CLOSE();
    });
    // ---- h += o2 W_o2 + b_o2
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) SI_WO_BLOCK(nb, xop, t_bo2)
  }
#undef SI_WO_BLOCK

  // ---- LN3
  layer_norm_row(t_g, t_b);

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

  // Slice-out.  Fast path (window rows, window start and frame size multiples of 8 positions):
  // each wavefront transposes its 32 tokens x 32 channels through a private LDS patch so that a lane
  // owns 8 consecutive positions of one channel -- one 16-byte load of x and one 16-byte store of
  // out; the x loads are issued two blocks ahead of their use.  Otherwise: element-wise.
  const Window& w = a.win;
  const int64_t cs = (int64_t)w.F * w.P;
  const bool vec_ok = (w.Pw % 8 == 0) && (w.p0 % 8 == 0) && (w.P % 8 == 0);
  // element-wise path: this lane's token
  const int64_t mm = live ? m : 0;
  const int mmi = (int)mm;  // window tokens fit 31 bits: 32-bit divisions
  const int64_t off0 = ((int64_t)(mmi / w.Pw / w.Fw) * w.C * w.F + (w.f0 + (mmi / w.Pw) % w.Fw)) * w.P + w.p0 + mmi % w.Pw;
  // vector path: lane-op i in {0,1} -> channel row r_i of the block, token group tg_i (8 tokens)
  int vr[2];
  int64_t voff[2];
  bool vlive[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = lane + kWave * i, tg = idx % 4;
    vr[i] = idx / 4;
    const int64_t m8 = (int64_t)blockIdx.x * 128 + wave * 32 + 8 * tg;
    vlive[i] = vec_ok && m8 < a.M;
    const int64_t mq = vlive[i] ? m8 : 0;
    const int mqi = (int)mq;
    voff[i] = ((int64_t)(mqi / w.Pw / w.Fw) * w.C * w.F + (w.f0 + (mqi / w.Pw) % w.Fw)) * w.P + w.p0 + mqi % w.Pw + (int64_t)vr[i] * cs;
  }
  u32x4_t xq[3][2];
  // every wavefront issues both loads (dead lanes read the tensor's first bytes): the step-closing
  // wait counts outstanding loads
#define SI_X_PREFETCH(nb)                                                                                  \
  if ((nb) < NB) {                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                          \
        xq[(nb) % 3][i] = *reinterpret_cast<const u32x4_t*>(a.x + (vlive[i] ? voff[i] + (int64_t)(32 * (nb)) * cs : 0)); \
  }
  SI_X_PREFETCH(0)
  SI_X_PREFETCH(1)

#define SI_PROJ_OUT_BLOCK(nb)                                                                    \
  {                                                                                              \
    f32x16_t y;                                                                                  \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) y[e] = 0.f;                                   \
    {                                                                                            \
      SI_STEP_OPEN();                                                                            \
      SI_X_PREFETCH((nb) + 2)                                                                    \
      _Pragma("unroll") for (int s = 0; s < SUB; ++s) {                                          \
        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SI_FRAG(s), hop[s], y, 0, 0, 0);             \
        SI_REFILL(s);                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                                       \
      }                                                                                          \
      SI_STEP_CLOSE_EXTRA((nb) + 2 < NB ? 2 : 0);                                                \
    }                                                                                            \
    if (vec_ok) {                                                                                \
      float(*patch)[36] = stage[wave];                                                           \
      _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
      _Pragma("unroll") for (int j = 0; j < 4; ++j)                                              \
        patch[8 * q + 4 * g + j][tcol] = y[4 * q + j] + t_bout[32 * (nb) + 8 * q + 4 * g + j];   \
      __builtin_amdgcn_wave_barrier();                                                           \
      _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                            \
        const float4 y0 = *reinterpret_cast<const float4*>(&patch[vr[i]][8 * ((lane + kWave * i) % 4)]);     \
        const float4 y1 = *reinterpret_cast<const float4*>(&patch[vr[i]][8 * ((lane + kWave * i) % 4) + 4]); \
        if (vlive[i]) {                                                                          \
          const u32x4_t xv = xq[(nb) % 3][i];                                                    \
          u32x4_t o;                                                                             \
          o.x = pack_bf16x2(__uint_as_float(xv.x << 16) + y0.x, __uint_as_float(xv.x & 0xffff0000u) + y0.y); \
          o.y = pack_bf16x2(__uint_as_float(xv.y << 16) + y0.z, __uint_as_float(xv.y & 0xffff0000u) + y0.w); \
          o.z = pack_bf16x2(__uint_as_float(xv.z << 16) + y1.x, __uint_as_float(xv.z & 0xffff0000u) + y1.y); \
          o.w = pack_bf16x2(__uint_as_float(xv.w << 16) + y1.z, __uint_as_float(xv.w & 0xffff0000u) + y1.w); \
          *reinterpret_cast<u32x4_t*>(a.out + voff[i] + (int64_t)(32 * (nb)) * cs) = o;          \
        }                                                                                        \
      }                                                                                          \
      __builtin_amdgcn_wave_barrier();                                                           \
    } else if (live) {                                                                           \
      _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                            \
        const int n = 32 * (nb) + 8 * q + 4 * g + j;                                             \
        const int64_t off = off0 + n * cs;                                                       \
        const float r = bf16_bits_to_float(a.x[off].v) + (y[4 * q + j] + t_bout[n]);             \
        a.out[off].v = float_to_bf16_bits(r);                                                    \
      }                                                                                          \
    }                                                                                            \
  }
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) SI_PROJ_OUT_BLOCK(nb)
#undef SI_X_PREFETCH
#undef SI_PROJ_OUT_BLOCK
#undef SI_SLOT
#undef SI_GELU_PACK
#undef SI_RUN_W2
#undef SI_RUN_W1
#undef SI_GEGLU_TAIL
#undef SI_REFILL
#undef SI_FRAG
#undef SI_STEP_CLOSE_EXTRA
#undef SI_STEP_CLOSE
#undef SI_STEP_OPEN
}

}  // namespace si
