// Spatial ResBlock operator group (GroupNorm, SiLU, 3x3 convolution) for bf16 features.  The
// convolution operands (normalised activations, bounded by construction, and the kernels) are held
// as fp16: the matrix cores run fp16 and bf16 at the same rate, and fp16's three extra significand
// bits keep the operand rounding of two chained 9*C-term contractions well inside the error budget
// that the final bf16 rounding of x + branch leaves.  bf16 kernels convert exactly unless a value
// lies outside fp16's normal range (|w| < 6.1e-5 rounds to a multiple of 2^-24, |w| > 65504 overflows).
// The resampling operators of the same group (stride-2 convolution, nearest doubling + convolution)
// run on the raw bf16 feature with bf16 operands (exact).
//   ring_mma_kernel      3x3 convolution, zero padding 1 -- same map, stride 2, or after nearest
//                           doubling -- as an implicit GEMM on the matrix cores; both operands arrive
//                           in MFMA fragment order by direct global->LDS loads through a multi-stage
//                           ring                                                             [MFMA bound]
//                           With one tap on one-pixel images (ntaps = 1, H = W = 1) the same kernel
//                           is a plain GEMM over M tokens: the transformer blocks' projections and
//                           FFN use it that way on fragment-order operands (weights packed by
//                           pack_transpose16_kernel, k_norm.h).
//   pack_conv_kernel        [O, C, 3, 3] bf16 kernel -> fragment stream in the order the kernel reads
//   temb_proj_kernel        e[b, o] = b_t[o] + sum_k SiLU(temb[b, k]) * W_t[k, o]
//   window_to_tokens_silu_kernel  slice window -> SiLU(GroupNorm1) (or a plain copy) -> operand in
//                           fragment order                                                   [HBM bound]
//   gn_partial_{tokens,frag}_kernel + gn_finish_tokens_kernel
//                           GroupNorm2 statistics per (image, group) of the fp16 intermediate,
//                           token-major or in fragment order
//   gn_silu_{tokens,frag}_kernel  SiLU(GroupNorm2(h)) -> fp16 operand in fragment order (in place
//                           when h already is)                                               [HBM bound]
#pragma once
#include <type_traits>
#include "si_common.h"
#include "k_gemm.h"

namespace si {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float silu(float v) { return v / (1.f + __expf(-v)); }

// Fragment order.  One fragment = 1 KiB = the 64 lanes' 16-byte operands of one
// v_mfma_f32_32x32x16_f16: lane l holds row l % 32 and the eight k-values 8*(l/32) .. +7.
//   activation  act_granule(t, c8) (k_norm.h): the 16 bytes (channels 8*c8 .. +7) of token t; fragments
//               are (32-token block, 16-channel step) pairs, 16-channel steps fastest.  The buffer starts
//               with a 256-byte block of zeros (what a tap outside the image reads).
//   weights     per (column tile, k-tile of 32 input channels of one tap): 2 k-steps x TN fragments,
//               rows = output channels; k-tiles ordered tap-major (tap = 3*(dy+1) + dx+1).

enum ConvMode { kConvSame = 0, kConvStride2 = 1, kConvNearestUp = 2 };

struct ConvArgs {
  const char* act;  // zero block + fragment-ordered 16-bit activation of the window (source map)
  const char* wf;   // fragment-ordered 16-bit kernel
  int64_t M;        // output tokens of the window; token m = img*H*W + y*W + x
  int C, O, H, W;   // input / output channels, output map
  int ncol, ntiles;  // column tiles, row tiles * column tiles
  int Hi, Wi;       // source map: (H, W) for kConvSame; the larger map for kConvStride2 (output pixel (y, x),
                    // tap (dy, dx) reads source (2y+dy, 2x+dx)); the smaller one for kConvNearestUp (reads
                    // source ((y+dy)/2, (x+dx)/2) when (y+dy, x+dx) lies inside the output map)
  int mode;
  int ntaps;        // 9, or 1: the centre tap only (a 1x1 convolution; the kernel stream then holds one tap)
  int col_major;    // tile order within an XCD's share: 0 = the column tiles of a row tile are neighbours (the
                    // activation rows stay in that XCD's L2, every XCD streams the whole kernel), 1 = the row
                    // tiles of a column tile are (the kernel columns stay, the activations stream): the
                    // operand that is streamed by all 8 XCDs should be the smaller one
};

// acc[m, o] = sum_{tap, c} a[m + dy*W + dx, c] * w[o, c, tap] over the taps whose source pixel lies
// inside the image.  Block = 4 wavefronts stacked along tokens; a wavefront owns TM*32 tokens x
// TN*32 output channels (weights as the MFMA row operand, tokens as columns: a lane ends up with 4
// consecutive output channels of one token, as in gemm_bf16_kernel).  A stage of the ring holds one
// k-tile (32 input channels of one tap): the wavefronts' activation fragments, gathered with the
// tap's shift by per-lane addresses, then the column tile's weight fragments.  Every wavefront
// issues the same number of loads per stage (a padding load repeats the wavefront's first weight
// fragment: same source, same destination) so that one s_waitcnt immediate closes a stage; stages
// beyond the last k-tile read the zero block into a slot nobody reads any more.  The loads are inline assembly (the compiler would otherwise wait for all of them
// before every LDS read); no compiler-visible vector-memory load sits inside the k loop.
// F16: operands are fp16 (v_mfma_f32_32x32x16_f16), else bf16 (v_mfma_f32_32x32x16_bf16).
// WS (wavefront-specialised, 512 threads): wavefronts 4..7 only feed the ring -- wavefront 4 + w issues
// exactly the loads wavefront w would issue -- and wavefronts 0..3 only read it and run the MFMAs, with
// the fragments of k-tile kt+1 read from LDS while the MFMAs of k-tile kt run.  The load issue of a
// stage (which blocks a wavefront while the address unit takes its KiB-sized requests) and the LDS
// latency then overlap with the MFMAs instead of preceding them, which is what a launch with one
// workgroup per CU at most lacks.  Both roles pass the same barriers: one per k-tile, then those of
// the epilogue.
template <class Epi, class = void>
struct epi_block32 : std::false_type {};
template <class Epi>
struct epi_block32<Epi, std::enable_if_t<Epi::kBlock32>> : std::true_type {};

template <int TM, int TN, int STAGES, bool F16, class Epi, bool WS = false>
__global__ __launch_bounds__(WS ? 512 : 256, (WS && TM * TN > 2) ? 1 : 2) void ring_mma_kernel(ConvArgs a, Epi epi) {
  constexpr int AF = 4 * TM * 2, WFR = 2 * TN;           // fragments per stage
  constexpr int NW = (WFR + 3) / 4;                      // weight loads per wavefront per stage
  constexpr int PER = 2 * TM + NW;                       // loads per wavefront per stage
  constexpr int SLOT = (AF + WFR) * 1024;
  static_assert((STAGES - 2) * PER <= 63, "vmcnt range");
  __shared__ __attribute__((aligned(1024))) char ring[STAGES * SLOT];

  // XCD-aware order: consecutive logical tiles (the column tiles of one row tile, then the next
  // row tile) stay on one XCD, whose L2 then serves the shared activation rows
  const int chunk = (a.ntiles + 7) / 8;
  const int tile = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
  if (tile >= a.ntiles) return;
  const int nrow = a.ntiles / a.ncol;
  const int col = a.col_major ? tile / nrow : tile % a.ncol;
  const int64_t m0 = (int64_t)(a.col_major ? tile % nrow : tile / a.ncol) * (128 * TM);

  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave_id = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wave = wave_id % 4;  // the quarter of the row tile this wavefront loads (feeding role) or contracts
  const bool producer = WS && wave_id >= 4;
  const int trow = lane % 32, half = lane / 32;
  const int P = a.H * a.W;
  const int per_tap = a.C / 32, nkt = a.ntaps * per_tap;

  int py[TM], px[TM];
  int64_t tok[TM], img0[TM];  // img0: first source token of the token's image
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    tok[j] = m0 + (wave * TM + j) * 32 + trow;
    if (P == 1 && a.Hi == 1 && a.Wi == 1) {  // a GEMM: one-pixel images, token m reads source token m (no 64-bit divisions)
      img0[j] = tok[j];
      py[j] = tok[j] < a.M ? 0 : -100000;
      px[j] = 0;
    } else {
      const int p = (int)(tok[j] % P);
      img0[j] = (tok[j] / P) * ((int64_t)a.Hi * a.Wi);
      py[j] = tok[j] < a.M ? p / a.W : -100000;  // far outside: no tap is ever inside
      px[j] = p % a.W;
    }
  }
  const unsigned ring_lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)ring;
  const char* wtile = a.wf + (int64_t)col * nkt * (WFR * 1024);

  unsigned tapv[TM];  // byte offset of the lane's granule for the current tap at channel 0, 0 = outside
  auto set_tap = [&](int tap) {
    const int t9 = a.ntaps == 1 ? 4 : tap;
    const int dy = t9 / 3 - 1, dx = t9 % 3 - 1;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      int sy, sx;
      bool in;
      if (a.mode == kConvStride2) {
        sy = 2 * py[j] + dy;
        sx = 2 * px[j] + dx;
        in = (unsigned)sy < (unsigned)a.Hi && (unsigned)sx < (unsigned)a.Wi;
      } else if (a.mode == kConvNearestUp) {
        in = (unsigned)(py[j] + dy) < (unsigned)a.H && (unsigned)(px[j] + dx) < (unsigned)a.W;
        sy = (py[j] + dy) >> 1;
        sx = (px[j] + dx) >> 1;
      } else {
        sy = py[j] + dy;
        sx = px[j] + dx;
        in = (unsigned)sy < (unsigned)a.Hi && (unsigned)sx < (unsigned)a.Wi;
      }
      const int64_t src = img0[j] + (int64_t)sy * a.Wi + sx;
      tapv[j] = in ? (unsigned)(kActZeroBytes + 16 * (((src >> 5) * (a.C / 16)) * 64 + half * 32 + (src & 31))) : 0u;
    }
  };
  int ld_tap = 0, ld_c = 0, ld_kt = 0;  // the k-tile the next issue() loads
  set_tap(0);
  auto issue = [&]() {
    const unsigned slot = ring_lds + (unsigned)((ld_kt % STAGES) * SLOT);
    const bool real = ld_kt < nkt;
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const unsigned voff = (real && tapv[j]) ? tapv[j] + (unsigned)((ld_c * 2 + ks) * 1024) : (unsigned)(lane * 16 % kActZeroBytes);
        const unsigned dst = slot + (unsigned)((((wave * TM + j) * 2 + ks)) * 1024);
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(a.act), "s"(dst) : "memory");
      }
    const char* wk = wtile + (int64_t)(real ? ld_kt : 0) * (WFR * 1024);
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const int fi = (wave + 4 * i) % WFR;  // beyond the stage's fragments: a repeat
      const char* sb = real ? wk + fi * 1024 : a.act;
      const unsigned voff = real ? (unsigned)(lane * 16) : (unsigned)(lane * 16 % kActZeroBytes);
      const unsigned dst = slot + (unsigned)((AF + fi) * 1024);
      asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(sb), "s"(dst) : "memory");
    }
    ++ld_kt;
    if (++ld_c == per_tap) {
      ld_c = 0;
      if (++ld_tap < a.ntaps) set_tap(ld_tap);
    }
  };

  f32x16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  constexpr int kWaitImm = (((STAGES - 2) * PER) & 0xF) | 0x70 | 0xF00 | ((((STAGES - 2) * PER) >> 4) << 14);
  struct Frags {
    u32x4_t wf[2][TN], af[2][TM];
  };
  auto read_frags = [&](int kt, Frags& f) {
    const char* slot = ring + (kt % STAGES) * SLOT;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < TN; ++i) f.wf[ks][i] = *reinterpret_cast<const u32x4_t*>(slot + (AF + ks * TN + i) * 1024 + lane * 16);
#pragma unroll
      for (int j = 0; j < TM; ++j) f.af[ks][j] = *reinterpret_cast<const u32x4_t*>(slot + ((wave * TM + j) * 2 + ks) * 1024 + lane * 16);
    }
  };
  auto contract = [&](const Frags& f) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          if constexpr (F16)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, f.wf[ks][i]),
                                                               __builtin_bit_cast(f16x8_t, f.af[ks][j]), acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, f.wf[ks][i]),
                                                                __builtin_bit_cast(bf16x8_t, f.af[ks][j]), acc[i][j], 0, 0, 0);
        }
  };
  if constexpr (WS) {
    if (producer) {
#pragma unroll
      for (int s = 0; s < STAGES - 1; ++s) issue();
      for (int kt = 0; kt < nkt; ++kt) {
        __builtin_amdgcn_s_waitcnt(kWaitImm);  // this wavefront's share of k-tile kt has landed
        __syncthreads();                       // barrier kt: every share has; k-tile kt-1's slot is no longer read
        issue();
      }
    } else {
      // barrier kt opens k-tile kt; its fragments are in registers (lgkmcnt(0)) before barrier kt+1 lets
      // the feeding wavefronts overwrite the slot two stages later
      constexpr int kLgkm0 = 0xC07F;  // lgkmcnt(0), other counters untouched
      Frags f0, f1;
      int kt = 0;
      if (nkt > 0) {
        __syncthreads();  // barrier 0
        read_frags(0, f0);
      }
      for (; kt + 2 <= nkt; kt += 2) {
        __builtin_amdgcn_s_waitcnt(kLgkm0);
        __syncthreads();  // barrier kt+1
        read_frags(kt + 1, f1);
        __builtin_amdgcn_sched_barrier(0);
        contract(f0);
        __builtin_amdgcn_s_waitcnt(kLgkm0);
        if (kt + 2 < nkt) {
          __syncthreads();  // barrier kt+2
          read_frags(kt + 2, f0);
        }
        __builtin_amdgcn_sched_barrier(0);
        contract(f1);
      }
      if (kt < nkt) contract(f0);  // odd count: the last k-tile was read behind barrier nkt-1
    }
  } else {
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue();
    for (int kt = 0; kt < nkt; ++kt) {
      // k-tile kt has landed for this wavefront once at most the STAGES-2 younger stages are in flight
      __builtin_amdgcn_s_waitcnt(kWaitImm);
      __syncthreads();  // ... and for every wavefront; all have also finished reading k-tile kt-1's slot
      issue();          // which the stage loaded now reuses
      Frags f;
      read_frags(kt, f);
      contract(f);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070 | 0xF00);  // vmcnt(0): the padding loads of the last stages

  if constexpr (Epi::kRows8) {
    // Output channels are far apart in the feature, tokens adjacent: hand the epilogue 8 consecutive
    // tokens of one channel.  One 32-channel block at a time is transposed through the (now idle)
    // ring: patch[channel][token], rows padded by 4 floats.
    constexpr int TOK = 128 * TM, LDP = TOK + 4;
    static_assert(32 * LDP * 4 <= STAGES * SLOT, "patch fits the ring");
    float* patch = reinterpret_cast<float*>(ring);
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      __syncthreads();  // the ring (first pass) or the previous block's patch is no longer read
      if (!producer) {
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) patch[(q * 8 + half * 4 + r) * LDP + (wave * TM + j) * 32 + trow] = acc[i][j][q * 4 + r];
      }
      __syncthreads();
      constexpr int NT = WS ? 512 : 256;  // the feeding wavefronts take their share of the stores
#pragma unroll
      for (int u = 0; u < 2 * TM * 256 / NT; ++u) {
        const int id = tid + u * NT, ch = id / (TOK / 8), t8 = (id % (TOK / 8)) * 8;
        const int n = (col * TN + i) * 32 + ch;
        const int64_t m = m0 + t8;
        if (n < a.O && m < a.M) {
          const float4 lo = *reinterpret_cast<const float4*>(patch + ch * LDP + t8);
          const float4 hi = *reinterpret_cast<const float4*>(patch + ch * LDP + t8 + 4);
          const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          epi.rows8(m, n, v, a.M);
        }
      }
    }
    return;
  }

  if (producer) return;
  if constexpr (epi_block32<Epi>::value) {
    // whole 32-column blocks go to the epilogue's block form (every lane takes part in its exchange)
    if (a.O % 32 == 0) {
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int i = 0; i < TN; ++i) {
          const int n0 = (col * TN + i) * 32;
          if (n0 < a.O) epi.block32(tok[j], tok[j] < a.M, n0, acc[i][j], half);
        }
      return;
    }
  }
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int64_t m = tok[j];
    if (m >= a.M) continue;
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = (col * TN + i) * 32 + q * 8 + half * 4;
        if (n < a.O) {
          const float v[4] = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
          epi(m, n, v);
        }
      }
    }
  }
}

// h[m, n] = fp16(acc + bias[n] + e[b(m), n])   (token-major; e may be NULL); b(m) = m / tokens_per_batch
struct EpiConvEmb {
  static constexpr bool kRows8 = false;
  _Float16* h;
  int64_t ld;
  const bf16* bias;
  const float* e;
  int64_t tokens_per_batch;
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    const float* er = e ? e + (int64_t)((int)m / (int)tokens_per_batch) * ld + n0 : nullptr;
    typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
    f16x4_t o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (_Float16)(v[i] + param_or(bias, n0 + i, 0.f) + (er ? er[i] : 0.f));
    *reinterpret_cast<f16x4_t*>(h + m * ld + n0) = o;
  }
};

// Same values, stored in the convolutions' fragment order (h points at the buffer's zero block):
// the lanes l and l+32 of a store fill the two halves of one 16-byte granule, a wavefront's store
// covers 32 consecutive granules.
struct EpiConvEmbFrag {
  static constexpr bool kRows8 = false;
  _Float16* h;
  int C;
  const bf16* bias;
  const float* e;
  int64_t tokens_per_batch;
  __device__ __forceinline__ void operator()(int64_t m, int n0, const float (&v)[4]) const {
    const float* er = e ? e + (int64_t)((int)m / (int)tokens_per_batch) * C + n0 : nullptr;
    typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
    f16x4_t o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (_Float16)(v[i] + param_or(bias, n0 + i, 0.f) + (er ? er[i] : 0.f));
    *reinterpret_cast<f16x4_t*>(h + kActZeroBytes / 2 + act_granule(m, n0 / 8, C) * 8 + (n0 % 8)) = o;
  }
};

// Slice-out of the ResBlock: out[b, n, f, p] = x[b, n, f, p] + acc + bias[n] for 8 consecutive tokens
// m .. m+7 of the window (token = (b*Fw + f - f0)*Pw + p); the sum is formed in fp32 and rounded once.
// 16-byte accesses when the eight tokens are eight aligned positions of one image.
struct EpiSliceOutRows {
  static constexpr bool kRows8 = true;
  const bf16* x;
  bf16* out;
  const bf16* bias;
  Window w;
  __device__ __forceinline__ void operator()(int64_t, int, const float (&)[4]) const {}
  __device__ __forceinline__ void rows8(int64_t m, int n, const float (&v)[8], int64_t M) const {
    const float bn = param_or(bias, n, 0.f);
    const int mi = (int)m;  // window tokens fit 31 bits: 32-bit divisions
    const int pl = mi % w.Pw;
    const int64_t bf = mi / w.Pw;
    const int64_t off = ((((int64_t)((int)bf / w.Fw)) * w.C + n) * w.F + (w.f0 + (int)bf % w.Fw)) * w.P + w.p0 + pl;
    if (pl + 7 < w.Pw && m + 7 < M && ((w.P | w.p0 | pl) & 7) == 0) {
      const uint4 raw = *reinterpret_cast<const uint4*>(x + off);
      const unsigned xw[4] = {raw.x, raw.y, raw.z, raw.w};
      unsigned ow[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float r0 = __uint_as_float(xw[i] << 16) + (v[2 * i] + bn);
        const float r1 = __uint_as_float(xw[i] & 0xffff0000u) + (v[2 * i + 1] + bn);
        ow[i] = (unsigned)float_to_bf16_bits(r0) | ((unsigned)float_to_bf16_bits(r1) << 16);
      }
      *reinterpret_cast<uint4*>(out + off) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int64_t mt = m + t;
        if (mt >= M) break;
        const int plt = (int)mt % w.Pw;
        const int64_t bft = (int)mt / w.Pw;
        const int64_t o2 = ((((int64_t)((int)bft / w.Fw)) * w.C + n) * w.F + (w.f0 + (int)bft % w.Fw)) * w.P + w.p0 + plt;
        out[o2] = from_float<bf16>(to_float(x[o2]) + (v[t] + bn));
      }
    }
  }
};

// out[b, n, f, p] = acc + bias[n] for 8 consecutive tokens of the window (no residual): the
// resampling operators' output.  Same addressing as EpiSliceOutRows, w describes the OUTPUT tensor.
struct EpiStoreRows {
  static constexpr bool kRows8 = true;
  bf16* out;
  const bf16* bias;
  Window w;
  __device__ __forceinline__ void operator()(int64_t, int, const float (&)[4]) const {}
  __device__ __forceinline__ void rows8(int64_t m, int n, const float (&v)[8], int64_t M) const {
    const float bn = param_or(bias, n, 0.f);
    const int mi = (int)m;  // window tokens fit 31 bits: 32-bit divisions
    const int pl = mi % w.Pw;
    const int64_t bf = mi / w.Pw;
    const int64_t off = ((((int64_t)((int)bf / w.Fw)) * w.C + n) * w.F + (w.f0 + (int)bf % w.Fw)) * w.P + w.p0 + pl;
    if (pl + 7 < w.Pw && m + 7 < M && ((w.P | w.p0 | pl) & 7) == 0) {
      unsigned ow[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        ow[i] = (unsigned)float_to_bf16_bits(v[2 * i] + bn) | ((unsigned)float_to_bf16_bits(v[2 * i + 1] + bn) << 16);
      *reinterpret_cast<uint4*>(out + off) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int64_t mt = m + t;
        if (mt >= M) break;
        const int plt = (int)mt % w.Pw;
        const int64_t bft = (int)mt / w.Pw;
        out[((((int64_t)((int)bft / w.Fw)) * w.C + n) * w.F + (w.f0 + (int)bft % w.Fw)) * w.P + w.p0 + plt] = from_float<bf16>(v[t] + bn);
      }
    }
  }
};

// Kernel [O, C, 3, 3] (bf16) -> fp16 (F16) or bf16 fragment stream for column tiles of TN*32 output channels:
// element e of lane l of fragment ((col*nkt + kt)*2 + ks)*TN + i is w[o, c, tap] with
// o = (col*TN + i)*32 + l%32, tap = kt / (C/32), c = (kt % (C/32))*32 + ks*16 + (l/32)*8 + e; rows
// beyond O are zero.  One thread per element.  Block 0 also clears the operand buffers' zero blocks.
template <bool F16>
__global__ __launch_bounds__(256) void pack_conv_kernel(const bf16* __restrict__ src, unsigned short* __restrict__ dst, int O, int C,
                                                        int TN, int ncol, unsigned* __restrict__ zero0, int zero_lanes = 0,
                                                        int64_t zero_lane_stride = 0, int64_t zero_pair = 0, int ntaps = 9) {
  // zero blocks of the operand buffers: one per lane (zero_lane_stride bytes apart), and, with
  // zero_pair, of a second buffer that many bytes further on in every lane
  if (blockIdx.x == 0 && threadIdx.x < kActZeroBytes / 4) {
    for (int l = 0; l < zero_lanes; ++l) {
      unsigned* z = zero0 + l * (zero_lane_stride / 4);
      z[threadIdx.x] = 0u;
      if (zero_pair) z[zero_pair / 4 + threadIdx.x] = 0u;
    }
  }
  const int per_tap = C / 32, nkt = ntaps * per_tap;  // ntaps == 1: src is [O, C]
  const int64_t total = (int64_t)ncol * nkt * 2 * TN * 512;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int e = (int)(idx % 8), l = (int)((idx / 8) % 64);
  int64_t f = idx / 512;
  const int i = (int)(f % TN); f /= TN;
  const int ks = (int)(f % 2); f /= 2;
  const int kt = (int)(f % nkt);
  const int col = (int)(f / nkt);
  const int o = (col * TN + i) * 32 + l % 32;
  const int tap = kt / per_tap, c = (kt % per_tap) * 32 + ks * 16 + (l / 32) * 8 + e;
  unsigned short bits = 0;
  if (o < O) {
    const bf16 v = src[((int64_t)o * C + c) * ntaps + tap];
    if constexpr (F16) bits = __builtin_bit_cast(unsigned short, (_Float16)to_float(v));
    else bits = v.v;
  }
  dst[idx] = bits;
}

// e[b, o] = b_t[o] + sum_k SiLU(temb[b, k]) * W_t[k, o].  One block (16 wavefronts) per (64 outputs,
// batch entry): wavefront q sums k = q, q+16, ... for output o = lane; the 16 partial sums are added
// in a fixed order.
__global__ __launch_bounds__(1024) void temb_proj_kernel(const bf16* __restrict__ temb, const bf16* __restrict__ wt,
                                                         const bf16* __restrict__ bt, float* __restrict__ e, int Kt, int O) {
  const int lane = threadIdx.x % kWave, q = threadIdx.x / kWave;
  const int o = blockIdx.x * kWave + lane;
  const int b = blockIdx.y;
  float s = 0.f;
  if (o < O) {
#pragma unroll 8
    for (int k = q; k < Kt; k += 16) s = fmaf(silu(to_float(temb[(int64_t)b * Kt + k])), to_float(wt[(int64_t)k * O + o]), s);
  }
  __shared__ float part[16][kWave];
  part[q][lane] = s;
  __syncthreads();
  if (q == 0 && o < O) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += part[i][lane];
    e[(int64_t)b * O + o] = t + param_or(bt, o, 0.f);
  }
}

// Second GroupNorm's statistics of the token-major fp16 feature h[img*P + p, c], in two steps so
// that every read is a full contiguous row:
//   gn_partial_tokens_kernel  block (chunk, img): per channel, sum and sum of squares of
//                             h - shift[c] over the chunk's kGnChunk tokens (shift[c] = the image's
//                             first token, so a common offset does not cancel in fp32);
//                             partial[((img*nchunk + chunk)*C + c)*2 + {0,1}]
//   gn_finish_tokens_kernel   block (img, group): merges chunks and the group's channels in fp64 in
//                             a fixed order; stats[(img*G + g)*2 + {0,1}] = {mean, 1/sqrt(var + eps)}
constexpr int kGnChunk = 64;

__global__ __launch_bounds__(256) void gn_partial_tokens_kernel(const _Float16* __restrict__ h, float* __restrict__ partial,
                                                                int P, int C) {
  const int chunk = blockIdx.x, img = blockIdx.y, nchunk = gridDim.x;
  const _Float16* base = h + (int64_t)img * P * C;
  const int p0 = chunk * kGnChunk;
  const int p1 = p0 + kGnChunk < P ? p0 + kGnChunk : P;
  for (int c = threadIdx.x; c < C; c += 256) {   // consecutive threads, consecutive channels: full rows
    const float shift = (float)base[c];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll 8
    for (int p = p0; p < p1; ++p) {
      const float d = (float)base[(int64_t)p * C + c] - shift;
      s1 += d;
      s2 = fmaf(d, d, s2);
    }
    float* o = partial + (((int64_t)img * nchunk + chunk) * C + c) * 2;
    o[0] = s1;
    o[1] = s2;
  }
}

__global__ __launch_bounds__(256) void gn_finish_tokens_kernel(const _Float16* __restrict__ h, const float* __restrict__ partial,
                                                               float* __restrict__ stats, int P, int C, int G, int nchunk,
                                                               float eps) {
  const int g = blockIdx.x % G, img = blockIdx.x / G;
  const int ng = C / G;
  const int lane = threadIdx.x % kWave, q = threadIdx.x / kWave;
  // lane < ng: one channel of the group (ng <= 64 is checked by the host); wavefront q takes chunks q, q+4, ...
  __shared__ double sh[2][4][kWave];
  double s1 = 0.0, s2 = 0.0;
  if (lane < ng) {
    const float2* src = reinterpret_cast<const float2*>(partial) + (int64_t)img * nchunk * C + g * ng + lane;
#pragma unroll 8
    for (int k = q; k < nchunk; k += 4) {
      const float2 v = src[(int64_t)k * C];
      s1 += (double)v.x;
      s2 += (double)v.y;
    }
  }
  sh[0][q][lane] = s1;
  sh[1][q][lane] = s2;
  __syncthreads();
  if (q != 0) return;
  double mean_c = 0.0, m2_c = 0.0;
  if (lane < ng) {
    s1 = (sh[0][0][lane] + sh[0][1][lane]) + (sh[0][2][lane] + sh[0][3][lane]);
    s2 = (sh[1][0][lane] + sh[1][1][lane]) + (sh[1][2][lane] + sh[1][3][lane]);
    const double n = (double)P;
    mean_c = (h ? (double)h[(int64_t)img * P * C + g * ng + lane] : 0.0) + s1 / n;  // h == NULL: sums were taken unshifted
    m2_c = s2 - s1 * s1 / n;   // sum of squared deviations from the channel's own mean
  }
  const double mean_g = wave_sum(lane < ng ? mean_c : 0.0) / (double)ng;
  const double dev = mean_c - mean_g;
  const double m2 = wave_sum(lane < ng ? m2_c + (double)P * dev * dev : 0.0);
  if (lane == 0) {
    double var = m2 / ((double)ng * (double)P);
    if (var < 0.0) var = 0.0;
    stats[(int64_t)blockIdx.x * 2 + 0] = (float)mean_g;
    stats[(int64_t)blockIdx.x * 2 + 1] = (float)(1.0 / sqrt(var + (double)eps));
  }
}

// a(m, c) = fp16(SiLU((h[m, c] - mean) * rstd * gamma[c] + beta[c])) in fragment order, four channels per thread
__global__ __launch_bounds__(256) void gn_silu_tokens_kernel(const _Float16* __restrict__ h, const float* __restrict__ stats,
                                                             const bf16* __restrict__ gamma, const bf16* __restrict__ beta,
                                                             _Float16* __restrict__ a, int64_t M, int P, int C, int G) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int cv = C / 4;
  if (idx >= M * cv) return;
  const int64_t m = idx / cv;
  const int c = (int)(idx % cv) * 4;
  const int64_t img = m / P;
  const int ng = C / G;
  typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
  const f16x4_t v = *reinterpret_cast<const f16x4_t*>(h + m * C + c);
  const float in[4] = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
  float o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int g = (c + i) / ng;
    const float mean = stats[(img * G + g) * 2 + 0], rstd = stats[(img * G + g) * 2 + 1];
    o[i] = silu((in[i] - mean) * rstd * param_or(gamma, c + i, 1.f) + param_or(beta, c + i, 0.f));
  }
  f16x4_t pk = {(_Float16)o[0], (_Float16)o[1], (_Float16)o[2], (_Float16)o[3]};
  *reinterpret_cast<f16x4_t*>(a + kActZeroBytes / 2 + act_granule(m, c / 8, C) * 8 + (c % 8)) = pk;
}

// The same two steps for an intermediate held in fragment order (P % 32 == 0: a 32-token block never
// straddles two images).  gn_partial_frag_kernel: block (chunk of kGnFragChunk token blocks, image,
// 64 channels); wavefront w owns the 16-channel step 4*blockIdx.z + w, a lane accumulates its 8
// channels over the chunk's token blocks (unshifted fp32 sums over at most 8 values per lane), the
// 32 lanes of each half are then summed by shuffles.  Output layout as gn_partial_tokens_kernel.
constexpr int kGnFragChunk = 8;

__global__ __launch_bounds__(256) void gn_partial_frag_kernel(const _Float16* __restrict__ h, float* __restrict__ partial, int P,
                                                              int C) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int chunk = blockIdx.x, img = blockIdx.y, nchunk = gridDim.x;
  const int cs = blockIdx.z * 4 + wave;
  if (cs >= C / 16) return;
  const int tb_img = P / 32;
  const int tb0 = chunk * kGnFragChunk;
  const int tb1 = tb0 + kGnFragChunk < tb_img ? tb0 + kGnFragChunk : tb_img;
  const f16x8_t* src = reinterpret_cast<const f16x8_t*>(h + kActZeroBytes / 2) + ((int64_t)img * tb_img * (C / 16) + cs) * 64 + lane;
  float s1[8], s2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0.f;
#pragma unroll
  for (int t = 0; t < kGnFragChunk; ++t) {
    if (tb0 + t < tb1) {
      const f16x8_t v = src[(int64_t)(tb0 + t) * (C / 16) * 64];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = (float)v[e];
        s1[e] += d;
        s2[e] = fmaf(d, d, s2[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
      s1[e] += __shfl_xor(s1[e], off);
      s2[e] += __shfl_xor(s2[e], off);
    }
  if (lane % 32 == 0) {
    float* o = partial + (((int64_t)img * nchunk + chunk) * C + cs * 16 + (lane / 32) * 8) * 2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o[2 * e] = s1[e];
      o[2 * e + 1] = s2[e];
    }
  }
}

// In place: granule (token, 8 channels) -> fp16(SiLU((h - mean) * rstd * gamma + beta)); one thread per granule.
__global__ __launch_bounds__(256) void gn_silu_frag_kernel(_Float16* __restrict__ h, const float* __restrict__ stats,
                                                           const bf16* __restrict__ gamma, const bf16* __restrict__ beta, int64_t M,
                                                           int P, int C, int G) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int lane = (int)(idx % 64);
  const int64_t frag = idx / 64;
  const int cs = (int)(frag % (C / 16));
  const int64_t token = (frag / (C / 16)) * 32 + lane % 32;
  if (token >= M) return;
  const int c0 = cs * 16 + (lane / 32) * 8;
  const int img = (int)(token / P);
  const int ng = C / G;
  f16x8_t* p = reinterpret_cast<f16x8_t*>(h + kActZeroBytes / 2) + idx;
  const f16x8_t v = *p;
  // the 8 channels lie in at most 8 consecutive groups; walk (group, position in group) instead of dividing per channel
  int g = c0 / ng, r = c0 - g * ng;
  const float2* st = reinterpret_cast<const float2*>(stats) + (int64_t)img * G;
  float2 mr = st[g];
  float ga[8], be[8];
  if (gamma) {
    const uint4 raw = *reinterpret_cast<const uint4*>(gamma + c0);
    const unsigned wv[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ga[2 * i] = __uint_as_float(wv[i] << 16);
      ga[2 * i + 1] = __uint_as_float(wv[i] & 0xffff0000u);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) ga[e] = 1.f;
  }
  if (beta) {
    const uint4 raw = *reinterpret_cast<const uint4*>(beta + c0);
    const unsigned wv[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      be[2 * i] = __uint_as_float(wv[i] << 16);
      be[2 * i + 1] = __uint_as_float(wv[i] & 0xffff0000u);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) be[e] = 0.f;
  }
  f16x8_t o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    o[e] = (_Float16)silu(((float)v[e] - mr.x) * mr.y * ga[e] + be[e]);
    if (++r == ng) {
      r = 0;
      ++g;
      if (e < 7) mr = st[g];
    }
  }
  *p = o;
}

// Slice-in of the ResBlock: a(m, c) = fp16(SiLU(GroupNorm1(x)[b, c, f, p])) in fragment order for the
// window's tokens m = (b*Fw + f - f0)*P + p.  64 x 64 (position x channel) tiles are transposed through LDS: 8-byte
// reads along positions, 16-byte writes along channels.  C % 8 == 0.
// RAW: no normalisation and no activation, the bf16 values are copied (operand of the resampling convolutions).
template <bool RAW>
__global__ __launch_bounds__(256) void window_to_tokens_silu_kernel(const bf16* __restrict__ x, const float* __restrict__ stats,
                                                                    const bf16* __restrict__ gamma, const bf16* __restrict__ beta,
                                                                    unsigned short* __restrict__ a, Window w) {
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
      float mean = 0.f, ga = 1.f, be = 0.f;
      if constexpr (!RAW) {
        const int g = c / ng;
        mean = stats[(((int64_t)b * w.F + f) * w.G + g) * 2 + 0];
        ga = param_or(gamma, c, 1.f) * stats[(((int64_t)b * w.F + f) * w.G + g) * 2 + 1];
        be = param_or(beta, c, 0.f);
      }
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
      for (int j = 0; j < 4; ++j) v[j] = RAW ? xv[j] : silu((xv[j] - mean) * ga + be);
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
      typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
      u16x8_t o;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if constexpr (RAW) o[j] = float_to_bf16_bits(tile[co + j][pl]);
        else o[j] = __builtin_bit_cast(unsigned short, (_Float16)tile[co + j][pl]);
      }
      *reinterpret_cast<u16x8_t*>(a + kActZeroBytes / 2 + act_granule((int64_t)bf * w.Pw + p, c / 8, w.C) * 8) = o;
    }
  }
}

}  // namespace si
