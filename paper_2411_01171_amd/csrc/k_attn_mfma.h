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
  const bf16* q;   // query i of sequence s: row s*Nq + i, head h at columns [64h, 64h+64); pre-scaled by
                   // softmax scale * log2(e), so that q k^T is the exponent in base 2
  int64_t ldq;
  const bf16* k;   // key j of key sequence ks = s / kv_div: row ks*Nk + j
  int64_t ldk;
  const bf16* vt;  // values, transposed: [ks][heads*64][Nkp], keys contiguous, Nkp % 8 == 0, zero padded
  bf16* o;         // output rows like q's
  int64_t ldo;
  int Nq, Nk, Nkp, heads, kv_div;
  int o_frag;        // 0: o rows of ldo elements; else o is a fragment-order buffer of that many channels per token
  int nqt, ntiles;   // query tiles per (sequence, head) pair; nqt * heads * sequences * ksplit (the grid is 8 * ceil(ntiles / 8))
  // FRAGIN only.  ksplit == 2: a workgroup takes one half of the keys; half kh leaves its output,
  // normalised by its own row sum, in o (kh = 0) / o2 (kh = 1) and, per lane, (reference maximum,
  // row sum) in ml[(kh * tiles + tile) * 64 + lane] -- whoever reads o merges the halves.
  int ksplit;
  bf16* o2;
  float2* ml;
  int64_t tiles32;   // 32-query tiles of all sequences
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

// Online softmax, per 32-key tile of this wavefront's 32 queries.  The queries arrive pre-scaled by
// softmax scale * log2(e) (the projection's epilogue does it before its one rounding), so S^T is in
// base-2 exponent units.  `minit` holds -m (the lane's reference maximum) in all 16 registers and is
// the accumulator input of the first score MFMA of a tile: the result registers are s - m and go
// straight into v_exp_f32.  m is a *lazy* maximum: it is raised (and the output rescaled) only when
// some lane's partial row sum says that an exponent went beyond kLazyTrigger, so the steady state
// per tile is 16 exponentials, 8 conversions to bf16 pairs and 8 packed dot products for the row
// sum -- no maximum, no subtraction, no cross-lane traffic.  lsum is the lane's own half of the row
// sum (16 of a tile's 32 keys); the two halves meet once, after the last tile.
constexpr float kLazyTrigger = 256.f;  // 2^8: an exponential this large, or 16 of them each above 2^4

__device__ __forceinline__ float dot2_ones(unsigned packed_bf16x2, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, packed_bf16x2), __builtin_bit_cast(bf16x2_t, 0x3f803f80u), acc,
                                         false);
}

struct AttnState {
  f32x16_t oacc[2];  // O^T, two 32-channel blocks
  f32x16_t minit;    // -m in every register
  float lsum;
};

// keys >= Nk of the tile that starts at key0 get a score of -inf
__device__ __forceinline__ void attn_mask_tile(f32x16_t& sc, int key0, int Nk, int g) {
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int i = 8 * (e / 4) + 4 * g + (e % 4);
    const int key = key0 + 16 * (i / 16) + kappa16(i % 16);
    if (key >= Nk) sc[e] = -INFINITY;
  }
}

__device__ __forceinline__ void attn_exp_pack(const f32x16_t& sc, float delta, u32x4_t (&pk)[2], float& rs) {
  unsigned w[8];
#pragma unroll
  for (int e = 0; e < 16; e += 2) w[e / 2] = pack_bf16x2(__builtin_amdgcn_exp2f(sc[e] - delta), __builtin_amdgcn_exp2f(sc[e + 1] - delta));
  rs = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) rs = dot2_ones(w[i], rs);
  pk[0] = u32x4_t{w[0], w[1], w[2], w[3]};
  pk[1] = u32x4_t{w[4], w[5], w[6], w[7]};
}

// Probabilities of one tile (scores sc = s - m) as the bf16 column operand pk of O^T += V^T P^T.
// Rare path: the reference maximum rises by delta -- the output so far and the row sum shrink by
// 2^-delta, and score tiles that were already taken against the old reference (l0, l1, l2; NULL =
// none) move by -delta.
__device__ __forceinline__ void attn_softmax_tile(f32x16_t& sc, u32x4_t (&pk)[2], AttnState& st, f32x16_t* l0, f32x16_t* l1,
                                                  f32x16_t* l2) {
  float rs;
  attn_exp_pack(sc, 0.f, pk, rs);
  if (__builtin_amdgcn_ballot_w64(rs > kLazyTrigger) != 0) {
    float mx = sc[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));  // both halves of the row agree on the new reference
    const float delta = fmaxf(mx, 0.f);
    const float alpha = __builtin_amdgcn_exp2f(-delta);
    st.lsum *= alpha;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) st.oacc[b][e] *= alpha;
#pragma unroll
    for (int e = 0; e < 16; ++e) st.minit[e] -= delta;
    attn_exp_pack(sc, delta, pk, rs);
    f32x16_t* later[3] = {l0, l1, l2};
#pragma unroll
    for (int i = 0; i < 3; ++i)
      if (later[i]) {
#pragma unroll
        for (int e = 0; e < 16; ++e) (*later[i])[e] -= delta;
      }
  }
  st.lsum += rs;
}

// S^T of the stage's two tiles against minit; kf: the 8 K fragments (tile u: kf[4u .. 4u+3]).  The
// two chains are interleaved so that no MFMA waits for the one issued just before it.
__device__ __forceinline__ void attn_scores(const u32x4_t (&kf)[8], const bf16x8_t (&qop)[4], const f32x16_t& minit, f32x16_t (&sc)[2]) {
  sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[0]), qop[0], minit, 0, 0, 0);
  sc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[4]), qop[0], minit, 0, 0, 0);
#pragma unroll
  for (int s4 = 1; s4 < 4; ++s4) {
    sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[s4]), qop[s4], sc[0], 0, 0, 0);
    sc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[4 + s4]), qop[s4], sc[1], 0, 0, 0);
  }
}

// O^T += V^T P^T for tile u; vf: the stage's 8 V^T fragments (tile u, channel block b, k-step t: vf[4u + 2b + t])
__device__ __forceinline__ void attn_pv(const u32x4_t (&vf)[8], int u, const u32x4_t (&pk)[2], f32x16_t (&oacc)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int b = 0; b < 2; ++b)
      oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf[4 * u + 2 * b + t]), __builtin_bit_cast(bf16x8_t, pk[t]),
                                                        oacc[b], 0, 0, 0);
}

// FRAGIN: the operands arrive, and the output leaves, as MFMA fragments written by the register-
// resident kernels around this one (1 KiB = 64 lanes x 16 bytes each, so every load and store of a
// wavefront is one contiguous KiB).  Nq % (32 NW) == 0, Nk % 64 == 0, kv_div == 1.
//   q: [(sequence, head)][32-query tile][k-step 0..3]        lane (query r, half g): channels 16 ks + frag_k(g, e)
//   k: [(sequence, head)][64-key stage][16 fragments]        in the order of a stage's ring slot: 8 of K
//      (tile u, k-step: lane (key r, g), same channels), then 8 of V^T (tile u, block b, 16-key step t:
//      lane (channel r, g), keys 16 t + frag_k(g, e)) -- keys in natural order, no permutation: the
//      result registers of S^T, packed pairwise, are already in the k-order of these V^T fragments
//   o: [32-token tile][k-step 0 .. 4 heads - 1 over the block width]   the column operand of the next contraction
template <int NW, bool FRAGIN = false>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_mfma_kernel(AttnMfmaArgs a) {
  constexpr int NS = kAttnStages, FR = 16;  // fragments per stage: 8 of K (2 tiles x 4 k-steps), 8 of V^T (2 tiles x 2 blocks x 2 k-steps)
  constexpr int PER = FR / NW;              // stage loads per lane
  static_assert(NW == 4 || NW == 8, "wavefronts per workgroup");
  __shared__ u32x4_t ring[NS][FR * kWave];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int r = lane % 32, g = lane / 32;
  // XCD-aware order: workgroups go to the 8 XCDs round-robin, and every XCD has an L2 of its own.
  // The work list (query tiles of one (sequence, head) pair after the other) is cut into 8
  // contiguous chunks, one per XCD, so that the keys and values of a pair are fetched into one L2
  // (two for a pair that straddles a chunk boundary) instead of into all eight.
  const int chunk = (a.ntiles + 7) / 8;
  const int work = (int)(blockIdx.x % 8) * chunk + (int)(blockIdx.x / 8);
  if (work >= a.ntiles) return;
  const int ksplit = FRAGIN ? a.ksplit : 1;
  // work list: the query tiles of one (pair, key half) after the other
  const int qtile = work % a.nqt, kh = (work / a.nqt) % ksplit, pair = work / (a.nqt * ksplit);
  const int h = pair % a.heads, s = pair / a.heads, ks = s / a.kv_div;
  const int qi = (qtile * NW + wave) * 32 + r;
  const bool qvalid = qi < a.Nq;
  const int nst = (a.Nk + 63) / 64 / ksplit;  // stages of this workgroup (FRAGIN: Nk % (64 ksplit) == 0)
  const int nfull = FRAGIN ? nst : a.Nk / 64;  // stages without missing keys (Nkp >= Nk: their V^T groups are in-row too)

  // ---- stage loads: fragment ids wave + NW*i, i < PER.  id < 8: K, tile u = id / 4, k-step id % 4;
  // id >= 8: V^T, tile u = (id - 8) / 4, channel block ((id - 8) / 2) % 2, k-step id % 2.
  // Address = scalar base (stage, fragment) + per-lane byte offset; the ragged last stage clamps
  // per lane instead (keys past the end are masked, so what they load only has to be finite).
  const int kap = 16 * (r / 16) + kappa16(r % 16);
  const unsigned kvoff = FRAGIN ? (unsigned)(lane * 16) : (unsigned)(((int64_t)kap * a.ldk + 8 * g) * 2);
  const unsigned vvoff = FRAGIN ? (unsigned)(lane * 16) : (unsigned)(((int64_t)r * a.Nkp + 8 * g) * 2);
  // row-major operands (not FRAGIN): this (sequence, head)'s key rows and transposed value rows
  const char* kb = FRAGIN ? nullptr : reinterpret_cast<const char*>(a.k + (int64_t)ks * a.Nk * a.ldk + h * 64);
  const char* vb = FRAGIN ? nullptr : reinterpret_cast<const char*>(a.vt + ((int64_t)ks * a.heads * 64 + h * 64) * a.Nkp);
  // FRAGIN: the pair's stage blocks, 16 KiB per stage
  const char* fb = reinterpret_cast<const char*>(a.k) + ((int64_t)((ks * a.heads + h) * ksplit + kh) * nst) * (16 * 1024);
  // Full stages are issued in order, so every fragment's source is a running scalar pointer that
  // advances by a fixed stride per stage (64 key rows of K; 64 keys = 128 bytes of a V^T row), and
  // the ring slot is a running scalar too: a stage's loads cost a few scalar additions.
  const int64_t kstride = FRAGIN ? 16 * 1024 : (int64_t)64 * a.ldk * 2;
  const int64_t vstride = FRAGIN ? 16 * 1024 : 128;
  const char* kcur[PER / 2];
  const char* vcur[PER / 2];
  unsigned loff[PER];
#pragma unroll
  for (int i = 0; i < PER / 2; ++i) {
    const int idk = wave_s + NW * i, idv = wave_s + NW * (i + PER / 2), j = idv - 8;
    kcur[i] = FRAGIN ? fb + idk * 1024 : kb + ((int64_t)(32 * (idk / 4)) * a.ldk + 16 * (idk % 4)) * 2;
    vcur[i] = FRAGIN ? fb + idv * 1024 : vb + ((int64_t)(32 * ((j / 2) % 2)) * a.Nkp + 32 * (j / 4) + 16 * (idv % 2)) * 2;
    loff[i] = (unsigned)(idk * kWave * 16);
    loff[PER / 2 + i] = (unsigned)(idv * kWave * 16);
  }
  const unsigned ring_lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(&ring[0][0]);
  constexpr unsigned kSlotBytes = FR * kWave * 16;
  unsigned islot = ring_lds;  // LDS address of the slot the next issued stage lands in
  auto next_slot = [&]() { islot = islot + kSlotBytes == ring_lds + NS * kSlotBytes ? ring_lds : islot + kSlotBytes; };
  auto issue_full = [&]() {
#pragma unroll
    for (int i = 0; i < PER / 2; ++i) {
      // assembly for the same reason as in WeightPipe::issue: completion is awaited explicitly
      asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(kvoff), "s"(kcur[i]), "s"(islot + loff[i]) : "memory");
      kcur[i] += kstride;
    }
#pragma unroll
    for (int i = 0; i < PER / 2; ++i) {
      asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(vvoff), "s"(vcur[i]), "s"(islot + loff[PER / 2 + i]) : "memory");
      vcur[i] += vstride;
    }
    next_slot();
  };
  // the ragged last stage: per-lane clamped addresses
  auto issue_ragged = [&](int st) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int id = wave_s + NW * i;
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
      asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(islot + loff[i]) : "memory");
    }
    next_slot();
  };
  auto issue = [&](int st) {
    if (st < nfull) issue_full();
    else if (!FRAGIN && st < nst) issue_ragged(st);
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st) issue(st);

  // ---- this lane's query as column operand (head channels in natural order, as K's fragments)
  bf16x8_t qop[4];
  if constexpr (FRAGIN) {
    const u32x4_t* qf = reinterpret_cast<const u32x4_t*>(a.q) +
                        (((int64_t)(s * a.heads + h) * (a.Nq / 32) + qtile * NW + wave) * 4) * kWave + lane;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) qop[s4] = __builtin_bit_cast(bf16x8_t, qf[s4 * kWave]);
  } else {
    const bf16* qrow = a.q + ((int64_t)s * a.Nq + (qvalid ? qi : a.Nq - 1)) * a.ldq + h * 64 + 8 * g;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) qop[s4] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(qrow + 16 * s4));
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the query loads; nothing the compiler tracks stays pending in the loop

  AttnState as;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) as.oacc[b][e] = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) as.minit[e] = 0.f;
  as.lsum = 0.f;

  // own loads of stage st have landed (at most the batches of the next NS - 2 stages stay in flight),
  // then the barrier: stage st is visible to all and everybody has left stage st - 1, whose slot the
  // load issued next overwrites
  auto open_stage = [&](int st) {
    const int younger = nst - 1 - st;
    if (NS >= 4 && younger >= 2) __builtin_amdgcn_s_waitcnt(WeightPipe<4>::wait_imm(2 * PER));
    else if (younger >= 1) __builtin_amdgcn_s_waitcnt(WeightPipe<4>::wait_imm(PER));
    else __builtin_amdgcn_s_waitcnt(WeightPipe<4>::wait_imm(0));
    __syncthreads();
    issue(st + NS - 1);
  };

  // Software pipeline over stages: while the matrix cores form the scores of stage st, the vector
  // ALUs exponentiate the first tile of stage st - 1; O^T += V^T P^T of that tile then runs under the
  // exponentials of the second one.  The V^T fragments of a stage are taken out of LDS before the
  // next barrier, because that barrier frees their slot.
  u32x4_t kf[8], vf[8];
  f32x16_t scA[2], scB[2];  // scores of the previous / the new stage, roles alternating
  open_stage(0);
#pragma unroll
  for (int i = 0; i < 8; ++i) kf[i] = ring[0][i * kWave + lane];
#pragma unroll
  for (int i = 0; i < 8; ++i) vf[i] = ring[0][(8 + i) * kWave + lane];
  attn_scores(kf, qop, as.minit, scA);
  {  // the first tile sets the reference maximum (key 0 always exists, so it is finite)
    if (nfull == 0) {
      attn_mask_tile(scA[0], 0, a.Nk, g);
      attn_mask_tile(scA[1], 32, a.Nk, g);
    }
    float mx = scA[0][0];
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, scA[0][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      as.minit[e] = -mx;
      scA[0][e] -= mx;
      scA[1][e] -= mx;
    }
  }
  const u32x4_t* slot = ring[0];  // slot of the stage whose scores are being formed
  auto next_ring = [&]() { slot = slot + FR * kWave == &ring[0][0] + NS * FR * kWave ? &ring[0][0] : slot + FR * kWave; };
  // one stage: scores of stage st into scn while scp (stage st - 1) is exponentiated and multiplied into O^T
  auto stage_body = [&](int st, f32x16_t(&scp)[2], f32x16_t(&scn)[2]) {
    open_stage(st);
    next_ring();
#pragma unroll
    for (int i = 0; i < 8; ++i) kf[i] = slot[i * kWave + lane];
    u32x4_t pk[2];
    attn_scores(kf, qop, as.minit, scn);
    attn_softmax_tile(scp[0], pk, as, &scp[1], &scn[0], &scn[1]);
    attn_pv(vf, 0, pk, as.oacc);
    attn_softmax_tile(scp[1], pk, as, &scn[0], &scn[1], nullptr);
    attn_pv(vf, 1, pk, as.oacc);
#pragma unroll
    for (int i = 0; i < 8; ++i) vf[i] = slot[(8 + i) * kWave + lane];
  };
  // drain: the last stage's tiles (the only ones that can hold keys past the end)
  auto drain = [&](f32x16_t(&scp)[2]) {
    if (nfull < nst && nst > 1) {
      attn_mask_tile(scp[0], 64 * (nst - 1), a.Nk, g);
      attn_mask_tile(scp[1], 64 * (nst - 1) + 32, a.Nk, g);
    }
    u32x4_t pk[2];
    attn_softmax_tile(scp[0], pk, as, &scp[1], nullptr, nullptr);
    attn_pv(vf, 0, pk, as.oacc);
    attn_softmax_tile(scp[1], pk, as, nullptr, nullptr, nullptr);
    attn_pv(vf, 1, pk, as.oacc);
  };
  int st = 1;
  for (; st + 1 < nst; st += 2) {
    stage_body(st, scA, scB);
    stage_body(st + 1, scB, scA);
  }
  if (st < nst) {
    stage_body(st, scA, scB);
    drain(scB);
  } else {
    drain(scA);
  }
  const float lsum = as.lsum + __shfl_xor(as.lsum, 32, kWave);  // the two halves of the row
  f32x16_t(&oacc)[2] = as.oacc;

  // ---- O^T / l: register 4q + j of block b is head channel 32b + 8q + 4g + j of this lane's query
  if constexpr (FRAGIN) {
    const float inv = 1.0f / lsum;
    const int64_t tile = (int64_t)s * (a.Nq / 32) + qtile * NW + wave;
    u32x4_t* of = reinterpret_cast<u32x4_t*>(kh ? a.o2 : a.o) + (tile * (a.heads * 4) + 4 * h) * kWave + lane;
    if (ksplit > 1) a.ml[(((int64_t)kh * a.heads + h) * a.tiles32 + tile) * kWave + lane] = make_float2(-as.minit[0], lsum);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        u32x4_t v;
        v.x = pack_bf16x2(oacc[b][8 * hf + 0] * inv, oacc[b][8 * hf + 1] * inv);
        v.y = pack_bf16x2(oacc[b][8 * hf + 2] * inv, oacc[b][8 * hf + 3] * inv);
        v.z = pack_bf16x2(oacc[b][8 * hf + 4] * inv, oacc[b][8 * hf + 5] * inv);
        v.w = pack_bf16x2(oacc[b][8 * hf + 6] * inv, oacc[b][8 * hf + 7] * inv);
        of[(2 * b + hf) * kWave] = v;
      }
  } else if (qvalid) {
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
