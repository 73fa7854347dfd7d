// Matrix-core attention for long sequences (spatial self-attention over H*W positions, cross-
// attention over the context tokens): bf16, head dimension 64, online softmax in fp32.
//
// One workgroup = NW x 32 queries of one (sequence, head), NW = 4 or 8 wavefronts sharing the key /
// value stages; one wavefront = 32 queries, which stay the
// *column* operand of every MFMA (v_mfma_f32_32x32x16_bf16: lane l supplies column l%32, k-slots
// 8*(l/32) .. +7; a result lane holds column l%32 and, in register 4q + j, row 8q + 4*(l/32) + j):
//   S^T[key, query] = K Q^T      row operand: 32 keys x 16 head channels, straight from k's rows
//   O^T[chan, query] += V^T P^T  row operand: 32 head channels x 16 keys, from the transposed
//                                copy vt[seq][channel][key]; column operand: the softmax result
//                                registers of the lane, converted to bf16 -- no data movement.
// The second product wants its 16 keys in the order of the result registers (rows 4g+j, then
// 8+4g+j of each half), so the key rows of a 32-key tile are *loaded* in a permuted order (kappa
// below) that makes that order the natural one: every fragment, K and V^T alike, is 16 contiguous
// bytes per lane and goes to LDS with direct global->LDS loads, 64 keys (16 KiB) per stage through
// a ring of kAttnStages stages.  A softmax is invariant under the permutation.
#pragma once
#include "k_fused.h"

namespace si {

struct AttnMfmaArgs {
  const bf16* q;   // query i of sequence s: row s*Nq + i, head h at columns [64h, 64h+64)
  int64_t ldq;
  const bf16* k;   // key j of key sequence ks = s / kv_div: row ks*Nk + j
  int64_t ldk;
  const bf16* vt;  // values, transposed: [ks][heads*64][Nkp], keys contiguous, Nkp % 8 == 0, zero padded
  bf16* o;         // output rows like q's
  int64_t ldo;
  int Nq, Nk, Nkp, heads, kv_div;
  float scale_log2;  // softmax scale * log2(e)
  int o_frag;        // 0: o rows of ldo elements; else o is a fragment-order buffer of that many channels per token
};

constexpr int kAttnStages = 3;  // 48 KiB of LDS: three 4-wavefront workgroups per CU

// key (within its 16-key group) whose score lands in MFMA row f of the group
__host__ __device__ constexpr int kappa16(int f) { return f < 4 || f >= 12 ? f : (f < 8 ? f + 4 : f - 4); }

// dst[(s*D + c)*Nkp + n] = src[(s*N + n)*ld + col0 + c]; zero for N <= n < Nkp.
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16* __restrict__ src, int64_t ld, int col0, bf16* __restrict__ dst,
                                                          int N, int Nkp, int D) {
  __shared__ unsigned short tile[32][33];
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8
  const int n0 = blockIdx.x * 32, c0 = blockIdx.y * 32, s = blockIdx.z;
  for (int nn = ty; nn < 32; nn += 8) {
    const int n = n0 + nn, c = c0 + tx;
    tile[nn][tx] = (n < N && c < D) ? src[((int64_t)s * N + n) * ld + col0 + c].v : (unsigned short)0;
  }
  __syncthreads();
  for (int cc = ty; cc < 32; cc += 8) {
    const int n = n0 + tx, c = c0 + cc;
    if (n < Nkp && c < D) dst[((int64_t)s * D + c) * Nkp + n].v = tile[tx][cc];
  }
}

// One 64-key stage of the online softmax for this wavefront's 32 queries.  MASKED: keys >= Nk exist
// in the stage (the last, ragged one) and get a score of -inf.
template <bool MASKED>
__device__ __forceinline__ void attn_stage(const u32x4_t* slot, int lane, int g, int key0, int Nk, float c, const bf16x8_t (&qop)[4],
                                           f32x16_t (&oacc)[2], float& m, float& lsum) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    f32x16_t sc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, slot[(4 * u + s4) * kWave + lane]), qop[s4], sc, 0, 0, 0);
    if (MASKED) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int i = 8 * (e / 4) + 4 * g + (e % 4);
        const int key = key0 + 32 * u + 16 * (i / 16) + kappa16(i % 16);
        if (key >= Nk) sc[e] = -INFINITY;
      }
    }
    float mx = sc[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    // the running maximum moves in the first tiles and rarely afterwards: rescale only when some
    // lane's maximum grew (finite from the first tile on, which always holds a real key)
    if (__builtin_amdgcn_ballot_w64(mx > m) != 0) {
      const float mnew = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f((m - mnew) * c);
      lsum *= alpha;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[b][e] *= alpha;
      m = mnew;
    }
    const float mc = m * c;
    float pr[16], rs = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      pr[e] = __builtin_amdgcn_exp2f(fmaf(sc[e], c, -mc));
      rs += pr[e];
    }
    rs += __shfl_xor(rs, 32, kWave);
    lsum += rs;
    bf16x8_t pop[2];
    pop[0] = to_operand(&pr[0]);
    pop[1] = to_operand(&pr[8]);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, slot[(8 + 4 * u + 2 * b + t) * kWave + lane]),
                                                          pop[t], oacc[b], 0, 0, 0);
  }
}

template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 2) void attn_mfma_kernel(AttnMfmaArgs a) {
  constexpr int NS = kAttnStages, FR = 16;  // fragments per stage: 8 of K (2 tiles x 4 k-steps), 8 of V^T (2 tiles x 2 blocks x 2 k-steps)
  constexpr int PER = FR / NW;              // stage loads per lane
  static_assert(NW == 4 || NW == 8, "wavefronts per workgroup");
  __shared__ u32x4_t ring[NS][FR * kWave];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int r = lane % 32, g = lane / 32;
  const int h = blockIdx.y, s = blockIdx.z, ks = s / a.kv_div;
  const int qi = (blockIdx.x * NW + wave) * 32 + r;
  const bool qvalid = qi < a.Nq;
  const int nst = (a.Nk + 63) / 64;
  const int nfull = a.Nk / 64;  // stages without missing keys (Nkp >= Nk: their V^T groups are in-row too)

  // ---- stage loads: fragment ids wave + NW*i, i < PER.  id < 8: K, tile u = id / 4, k-step id % 4;
  // id >= 8: V^T, tile u = (id - 8) / 4, channel block ((id - 8) / 2) % 2, k-step id % 2.
  // Address = scalar base (stage, fragment) + per-lane byte offset; the ragged last stage clamps
  // per lane instead (keys past the end are masked, so what they load only has to be finite).
  const int kap = 16 * (r / 16) + kappa16(r % 16);
  const unsigned kvoff = (unsigned)(((int64_t)kap * a.ldk + 8 * g) * 2);
  const unsigned vvoff = (unsigned)(((int64_t)r * a.Nkp + 8 * g) * 2);
  const char* kb = reinterpret_cast<const char*>(a.k + (int64_t)ks * a.Nk * a.ldk + h * 64);
  const char* vb = reinterpret_cast<const char*>(a.vt + ((int64_t)ks * a.heads * 64 + h * 64) * a.Nkp);
  auto issue = [&](int st) {
    if (st < nst) {
      const unsigned dst = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(ring[st % NS]);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int id = wave_s + NW * i;  // scalar; K for i < PER / 2
        const unsigned l = dst + (unsigned)(id * kWave * 16);
        if (st < nfull) {
          const char* sb = i < PER / 2
                               ? kb + ((int64_t)(64 * st + 32 * (id / 4)) * a.ldk + 16 * (id % 4)) * 2
                               : vb + ((int64_t)(32 * (((id - 8) / 2) % 2)) * a.Nkp + 64 * st + 32 * ((id - 8) / 4) + 16 * (id % 2)) * 2;
          // assembly for the same reason as in WeightPipe::issue: completion is awaited explicitly
          asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(i < PER / 2 ? kvoff : vvoff), "s"(sb), "s"(l) : "memory");
        } else {
          const bf16* src;
          if (i < PER / 2) {
            int key = 64 * st + 32 * (id / 4) + kap;
            key = key < a.Nk ? key : a.Nk - 1;
            src = reinterpret_cast<const bf16*>(kb) + (int64_t)key * a.ldk + 16 * (id % 4) + 8 * g;
          } else {
            int k0 = 64 * st + 32 * ((id - 8) / 4) + 16 * (id % 2) + 8 * g;  // groups of 8 keys past the row's end hold masked keys only
            k0 = k0 < a.Nkp - 8 ? k0 : a.Nkp - 8;
            src = reinterpret_cast<const bf16*>(vb) + (int64_t)(32 * (((id - 8) / 2) % 2) + r) * a.Nkp + k0;
          }
          asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(l) : "memory");
        }
      }
    }
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st) issue(st);

  // ---- this lane's query as column operand (head channels in natural order, as K's fragments)
  bf16x8_t qop[4];
  {
    const bf16* qrow = a.q + ((int64_t)s * a.Nq + (qvalid ? qi : a.Nq - 1)) * a.ldq + h * 64 + 8 * g;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) qop[s4] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(qrow + 16 * s4));
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the query loads; nothing the compiler tracks stays pending in the loop

  f32x16_t oacc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[b][e] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const float c = a.scale_log2;

  for (int st = 0; st < nst; ++st) {
    // own loads of stage st have landed: at most the batches of the next NS - 2 stages stay in flight
    {
      const int younger = nst - 1 - st;
      if (NS >= 4 && younger >= 2) __builtin_amdgcn_s_waitcnt(WeightPipe<4>::wait_imm(2 * PER));
      else if (younger >= 1) __builtin_amdgcn_s_waitcnt(WeightPipe<4>::wait_imm(PER));
      else __builtin_amdgcn_s_waitcnt(WeightPipe<4>::wait_imm(0));
    }
    __syncthreads();  // stage st is visible to all; everybody has left stage st - 1, whose slot is loaded next
    issue(st + NS - 1);
    const u32x4_t* slot = ring[st % NS];
    if (st < nfull) attn_stage<false>(slot, lane, g, 64 * st, a.Nk, c, qop, oacc, m, lsum);
    else attn_stage<true>(slot, lane, g, 64 * st, a.Nk, c, qop, oacc, m, lsum);
  }

  // ---- O^T / l: register 4q + j of block b is head channel 32b + 8q + 4g + j of this lane's query
  if (qvalid) {
    const float inv = 1.0f / lsum;
    const int64_t m = (int64_t)s * a.Nq + qi;
    bf16* orow = a.o + m * a.ldo + h * 64 + 4 * g;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 v;
        v.x = pack_bf16x2(oacc[b][4 * q + 0] * inv, oacc[b][4 * q + 1] * inv);
        v.y = pack_bf16x2(oacc[b][4 * q + 2] * inv, oacc[b][4 * q + 3] * inv);
        bf16* dst = a.o_frag ? a.o + act_offset(m, h * 64 + 32 * b + 8 * q + 4 * g, a.o_frag) : orow + 32 * b + 8 * q;
        *reinterpret_cast<uint2*>(dst) = v;
      }
  }
}

}  // namespace si
