// Host side of the Spatial ResBlock operator group (see include/si.h): argument validation,
// workspace layout, the slice loop over frame windows and the kernel launches.  Part of the
// translation unit si_api.hip (uses its stage timing, alignment and overlap helpers).
#pragma once
#include "k_conv.h"

#ifndef SI_RES_LANES3_MIN
#define SI_RES_LANES3_MIN 12
#endif
#ifndef SI_CONV_BIG_MIN
#define SI_CONV_BIG_MIN 512
#endif

namespace si {

struct ResPlan {
  int B, C, F, H, W, G, Kt;
  int Co;              // output channels (== C: identity skip, else the 1x1 skip convolution runs)
  int TN, ncol;        // column tiles of the convolution kernel: ncol tiles of TN*32 output channels
  int64_t P, slice_len, Mmax;
  int lanes;           // frame windows in flight (two streams) when there are many small ones
  size_t lane_stride;
  size_t off_stats, off_emb, off_a, off_xr, off_h, off_stats2, off_part, off_w1, off_w2, off_wskip;
  size_t weights_bytes, total_bytes;
};

static void conv_column_tiles(int O, int64_t rows_in_flight, int* TN, int* ncol);

static si_status make_res_plan(const si_tensor5* x, const si_resblock_weights* w, int64_t slice_len, ResPlan* p) {
  if (!x || !w) return SI_ERR_NULL;
  if (x->dtype != SI_BF16) return SI_ERR_DTYPE;
  if (x->B < 1 || x->C < 1 || x->F < 1 || x->H < 1 || x->W < 1) return SI_ERR_SHAPE;
  if (w->gn_groups < 1 || x->C % w->gn_groups || x->C % 32 || x->C > 8192) return SI_ERR_SHAPE;
  if (x->C / w->gn_groups > 64) return SI_ERR_SHAPE;  // a group's channels are merged by one wavefront
  const int64_t P = x->H * x->W;
  if (x->B > 65535 || x->F > 65535 || x->H > 4096 || x->W > 4096) return SI_ERR_SHAPE;
  if ((double)x->B * x->C * x->F * (double)P >= 1099511627776.0) return SI_ERR_SHAPE;
  if ((int64_t)(x->C / w->gn_groups) * P >= (1LL << 31)) return SI_ERR_SHAPE;
  if (!(w->gn_eps >= 0.f)) return SI_ERR_ARG;
  if (w->temb_dim < 0 || w->temb_dim > 65536) return SI_ERR_SHAPE;
  if (slice_len < 1) return SI_ERR_SLICE;
  p->B = (int)x->B; p->C = (int)x->C; p->F = (int)x->F; p->H = (int)x->H; p->W = (int)x->W;
  p->G = w->gn_groups; p->Kt = w->temb_dim; p->P = P;
  p->Co = w->c_out > 0 ? w->c_out : p->C;
  if (p->Co % w->gn_groups || p->Co % 32 || p->Co > 8192 || p->Co / w->gn_groups > 64) return SI_ERR_SHAPE;
  if ((double)x->B * p->Co * x->F * (double)P >= 1099511627776.0) return SI_ERR_SHAPE;
  p->slice_len = slice_len < x->F ? slice_len : x->F;
  p->Mmax = (int64_t)x->B * p->slice_len * P;
  if (p->Mmax >= (1LL << 31) / 16) return SI_ERR_SHAPE;
  const size_t C = (size_t)p->C, Co = (size_t)p->Co;
  const bool skip_conv = p->Co != p->C;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  p->off_stats = take((size_t)p->B * p->F * p->G * 2 * sizeof(float));
  p->off_emb = take((size_t)p->B * Co * sizeof(float));
  // one window's intermediates: the fp16 operand of either convolution, the fp16 output of the first
  // one, the second GroupNorm's statistics
  if ((double)p->Mmax * (double)(C > Co ? C : Co) * 2.0 + 4096.0 >= 4294967296.0) return SI_ERR_SHAPE;  // 32-bit operand offsets
  const size_t Mpad = (size_t)((p->Mmax + 31) / 32 * 32);
  p->off_a = take(kActZeroBytes + Mpad * (C > Co ? C : Co) * 2);   // conv1's operand; conv2's when h is token-major
  p->off_xr = take(skip_conv ? kActZeroBytes + Mpad * C * 2 : 0);  // the raw window, operand of the 1x1 skip
  p->off_h = take(kActZeroBytes + Mpad * Co * 2);                   // token-major or fragment order
  p->off_stats2 = take((size_t)p->B * p->slice_len * p->G * 2 * sizeof(float));
  p->off_part = take((size_t)p->B * p->slice_len * (size_t)((P + 31) / 32) * Co * 2 * sizeof(float));  // >= either chunking
  const int64_t n_slices = (p->F + p->slice_len - 1) / p->slice_len;
  // windows in flight: their buffers together stay within a quarter of the unsliced ones
  p->lanes = n_slices >= SI_RES_LANES3_MIN ? 3 : n_slices >= 8 ? 2 : 1;
  p->lane_stride = off - p->off_a;
  for (int l = 1; l < p->lanes; ++l) take(p->lane_stride);
  const size_t act_end = off;
  conv_column_tiles(p->Co, (p->Mmax + 127) / 128 * p->lanes, &p->TN, &p->ncol);
  const size_t per_ktile = (size_t)p->ncol * 2 * p->TN * 1024;  // bytes of one 32-channel k-tile over all column tiles
  p->off_w1 = take(per_ktile * 9 * (C / 32));
  p->off_w2 = take(per_ktile * 9 * (Co / 32));
  p->off_wskip = take(skip_conv ? per_ktile * (C / 32) : 0);
  p->weights_bytes = off - act_end;
  p->total_bytes = off;
  return SI_OK;
}

template <int TM, int TN, int STAGES, bool F16, class Epi>
static void launch_conv_tile(const ConvArgs& a, Epi epi, hipStream_t st) {
  const int grid = (a.ntiles + 7) / 8 * 8;
  ring_mma_kernel<TM, TN, STAGES, F16, Epi><<<grid, 256, 0, st>>>(a, epi);
}

// Column tiles of the convolution kernel: the candidate width that pads the output channels least,
// the wider one on a tie.  rows_in_flight = 128-token row tiles of the windows in flight: while the
// launches together leave CUs without a workgroup, a narrower tile (4 or 2 blocks of 32 channels,
// never one: measured slower throughout) that pads at most a tenth more takes its place (down-
// sampling of a 72 x 128 map at 320 channels: 2 x 72 workgroups of 160 channels -> 2 x 180 of 64).
static void conv_column_tiles(int O, int64_t rows_in_flight, int* TN, int* ncol) {
  *TN = 1;
  *ncol = (O + 31) / 32;
  for (int tn : {2, 4, 5}) {
    const int nc = (O + 32 * tn - 1) / (32 * tn);
    if (nc * tn <= *ncol * *TN) {
      *TN = tn;
      *ncol = nc;
    }
  }
  for (int tn : {4, 2}) {
    if (rows_in_flight * *ncol >= 256) break;
    if (tn >= *TN) continue;
    const int nc = (O + 32 * tn - 1) / (32 * tn);
    if (nc * tn * 10 <= *ncol * *TN * 11) {
      *TN = tn;
      *ncol = nc;
    }
  }
}

// Row tiles of 256 tokens when that still gives every CU two blocks, else 128 tokens.  M output
// tokens on an H x W map; (Hi, Wi, mode) describe the source map (see ConvArgs).
template <bool F16, class Epi>
static si_status launch_conv3x3(const char* stage, const void* act, const void* wf, int64_t M, int C, int TN, int ncol, int H,
                                int W, int Hi, int Wi, int mode, Epi epi, hipStream_t st, int O = 0, int ntaps = 9) {
  StageScope scope(stage, st);
  ConvArgs a{static_cast<const char*>(act), static_cast<const char*>(wf), M, C, O ? O : C, H, W, ncol, 0, Hi, Wi, mode, ntaps};
  const int64_t rows2 = (M + 255) / 256;
  const bool big = rows2 * ncol >= SI_CONV_BIG_MIN;
  a.ntiles = (int)((big ? rows2 : (M + 127) / 128) * ncol);
  switch (TN * 2 + (big ? 1 : 0)) {
    case 11: launch_conv_tile<2, 5, 3, F16>(a, epi, st); break;
    case 10: launch_conv_tile<1, 5, 4, F16>(a, epi, st); break;
    case 9: launch_conv_tile<2, 4, 3, F16>(a, epi, st); break;
    case 8: launch_conv_tile<1, 4, 4, F16>(a, epi, st); break;
    case 5: launch_conv_tile<2, 2, 4, F16>(a, epi, st); break;
    case 4: launch_conv_tile<1, 2, 4, F16>(a, epi, st); break;
    case 3: launch_conv_tile<2, 1, 4, F16>(a, epi, st); break;
    case 2: launch_conv_tile<1, 1, 4, F16>(a, epi, st); break;
    default: return SI_ERR_SHAPE;
  }
  SI_CHECK_LAUNCH();
  return SI_OK;
}

static si_status run_resblock(const ResPlan& p, const si_tensor5* x, const si_resblock_weights* w, const void* temb,
                              si_tensor5* out, char* ws, hipStream_t st0) {
  const bf16* X = static_cast<const bf16*>(x->ptr);
  bf16* OUT = static_cast<bf16*>(out->ptr);
  float* stats = reinterpret_cast<float*>(ws + p.off_stats);
  float* emb = p.Kt ? reinterpret_cast<float*>(ws + p.off_emb) : nullptr;
  _Float16* w1 = reinterpret_cast<_Float16*>(ws + p.off_w1);
  _Float16* w2 = reinterpret_cast<_Float16*>(ws + p.off_w2);
  unsigned short* wskip = reinterpret_cast<unsigned short*>(ws + p.off_wskip);
  const int C = p.C, Co = p.Co;
  const bool skip_conv = Co != C;
  auto cB = [](const void* q) { return static_cast<const bf16*>(q); };

  // ---- once per call: kernel re-layout, embedding projection, first GroupNorm's statistics
  {
    StageScope scope("pack_weights", st0);
    const int64_t per_ktile = (int64_t)p.ncol * 2 * p.TN * 512;  // elements of one k-tile over all column tiles
    auto blocks = [&](int64_t elems) { return (unsigned)((elems + 255) / 256); };
    unsigned* z0 = reinterpret_cast<unsigned*>(ws + p.off_a);
    pack_conv_kernel<true><<<blocks(per_ktile * 9 * (C / 32)), 256, 0, st0>>>(cB(w->w_conv1), reinterpret_cast<unsigned short*>(w1),
                                                                             Co, C, p.TN, p.ncol, z0, p.lanes,
                                                                             (int64_t)p.lane_stride, (int64_t)(p.off_h - p.off_a));
    SI_CHECK_LAUNCH();
    pack_conv_kernel<true><<<blocks(per_ktile * 9 * (Co / 32)), 256, 0, st0>>>(cB(w->w_conv2), reinterpret_cast<unsigned short*>(w2),
                                                                              Co, Co, p.TN, p.ncol, nullptr);
    SI_CHECK_LAUNCH();
    if (skip_conv) {
      pack_conv_kernel<false><<<blocks(per_ktile * (C / 32)), 256, 0, st0>>>(cB(w->w_skip), wskip, Co, C, p.TN, p.ncol,
                                                                            reinterpret_cast<unsigned*>(ws + p.off_xr), p.lanes,
                                                                            (int64_t)p.lane_stride, 0, 1);
      SI_CHECK_LAUNCH();
    }
    if (emb) {
      temb_proj_kernel<<<dim3((unsigned)((Co + 63) / 64), (unsigned)p.B), 1024, 0, st0>>>(cB(temb), cB(w->w_temb),
                                                                                           cB(w->b_temb), emb, p.Kt, Co);
      SI_CHECK_LAUNCH();
    }
  }
  {
    StageScope scope("gn_stats", st0);
    const unsigned blocks = (unsigned)(p.B * p.F * p.G);
    if (p.P % 8 == 0) gn_stats_kernel<bf16, 8><<<blocks, 256, 0, st0>>>(X, stats, C, p.F, p.P, p.G, w->gn_eps);
    else gn_stats_kernel<bf16, 1><<<blocks, 256, 0, st0>>>(X, stats, C, p.F, p.P, p.G, w->gn_eps);
    SI_CHECK_LAUNCH();
  }

  AuxStream* aux = nullptr;
  const int lanes = g_timing ? 1 : p.lanes;  // per-stage timing: one window at a time
  if (lanes >= 2) {
    SI_TRY(aux_stream(&aux));
    SI_TRY(lanes_fork(aux, lanes, st0));
  }

  // ---- the frame windows (Sec. 4.1): each goes through the whole group and lands in its window of out
  int widx = 0;
  for (int64_t f0 = 0; f0 < p.F; f0 += p.slice_len, ++widx) {
    const int lane_id = widx % lanes;
    hipStream_t st = lane_id == 0 ? st0 : aux->s[lane_id - 1];
    char* lane_ws = ws + (size_t)lane_id * p.lane_stride;
    _Float16* a = reinterpret_cast<_Float16*>(lane_ws + p.off_a);
    _Float16* h = reinterpret_cast<_Float16*>(lane_ws + p.off_h);
    float* stats2 = reinterpret_cast<float*>(lane_ws + p.off_stats2);
    float* part = reinterpret_cast<float*>(lane_ws + p.off_part);
    const int Fw = (int)((f0 + p.slice_len <= p.F) ? p.slice_len : p.F - f0);
    const int64_t M = (int64_t)p.B * Fw * p.P;
    Window win{p.B, C, p.F, p.P, (int)f0, Fw, 0, (int)p.P, p.G};
    {
      StageScope scope("slice_in", st);
      dim3 grid((unsigned)((p.P + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)(p.B * Fw));
      window_to_tokens_silu_kernel<false><<<grid, 256, 0, st>>>(X, stats, cB(w->gn1_g), cB(w->gn1_b),
                                                                reinterpret_cast<unsigned short*>(a), win);
      SI_CHECK_LAUNCH();
    }
    Window win_out{p.B, Co, p.F, p.P, (int)f0, Fw, 0, (int)p.P, p.G};
    if (skip_conv) {  // out window := w_skip x + b_skip; conv2's epilogue then adds the branch in place
      unsigned short* xr = reinterpret_cast<unsigned short*>(lane_ws + p.off_xr);
      {
        StageScope scope("slice_in_raw", st);
        dim3 grid((unsigned)((p.P + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)(p.B * Fw));
        window_to_tokens_silu_kernel<true><<<grid, 256, 0, st>>>(X, nullptr, nullptr, nullptr, xr, win);
        SI_CHECK_LAUNCH();
      }
      EpiStoreRows epi{OUT, cB(w->b_skip), win_out};
      SI_TRY(launch_conv3x3<false>("conv_skip", xr, wskip, M, C, p.TN, p.ncol, p.H, p.W, p.H, p.W, kConvSame, epi, st, Co, 1));
    }
    // The intermediate between the convolutions stays in fragment order when no 32-token block
    // straddles two images: GroupNorm2 + SiLU then run in place on it and conv2 reads it as it is.
    const bool frag_h = p.P % 32 == 0;
    if (frag_h) {
      EpiConvEmbFrag epi{h, Co, cB(w->b_conv1), emb, (int64_t)Fw * p.P};
      SI_TRY(launch_conv3x3<true>("conv1", a, w1, M, C, p.TN, p.ncol, p.H, p.W, p.H, p.W, kConvSame, epi, st, Co));
    } else {
      EpiConvEmb epi{h, (int64_t)Co, cB(w->b_conv1), emb, (int64_t)Fw * p.P};
      SI_TRY(launch_conv3x3<true>("conv1", a, w1, M, C, p.TN, p.ncol, p.H, p.W, p.H, p.W, kConvSame, epi, st, Co));
    }
    {
      StageScope scope("gn2_stats", st);
      if (frag_h) {
        const int nchunk = (int)((p.P / 32 + kGnFragChunk - 1) / kGnFragChunk);
        gn_partial_frag_kernel<<<dim3((unsigned)nchunk, (unsigned)(p.B * Fw), (unsigned)((Co / 16 + 3) / 4)), 256, 0, st>>>(
            h, part, (int)p.P, Co);
        SI_CHECK_LAUNCH();
        gn_finish_tokens_kernel<<<(unsigned)(p.B * Fw * p.G), 256, 0, st>>>(nullptr, part, stats2, (int)p.P, Co, p.G, nchunk,
                                                                            w->gn_eps);
      } else {
        const int nchunk = (int)((p.P + kGnChunk - 1) / kGnChunk);
        gn_partial_tokens_kernel<<<dim3((unsigned)nchunk, (unsigned)(p.B * Fw)), 256, 0, st>>>(h, part, (int)p.P, Co);
        SI_CHECK_LAUNCH();
        gn_finish_tokens_kernel<<<(unsigned)(p.B * Fw * p.G), 256, 0, st>>>(h, part, stats2, (int)p.P, Co, p.G, nchunk, w->gn_eps);
      }
      SI_CHECK_LAUNCH();
    }
    {
      StageScope scope("gn2_silu", st);
      if (frag_h) {
        const int64_t n = (M + 31) / 32 * (Co / 16) * 64;
        gn_silu_frag_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(h, stats2, cB(w->gn2_g), cB(w->gn2_b), M, (int)p.P, Co, p.G);
      } else {
        const int64_t n = M * (Co / 4);
        gn_silu_tokens_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(h, stats2, cB(w->gn2_g), cB(w->gn2_b), a, M, (int)p.P,
                                                                           Co, p.G);
      }
      SI_CHECK_LAUNCH();
    }
    {
      // residual source: x itself, or the skip convolution's result already sitting in the out window
      EpiSliceOutRows epi{skip_conv ? OUT : X, OUT, cB(w->b_conv2), win_out};
      SI_TRY(launch_conv3x3<true>("conv2", frag_h ? h : a, w2, M, Co, p.TN, p.ncol, p.H, p.W, p.H, p.W, kConvSame, epi, st));
    }
  }
  if (lanes >= 2) SI_TRY(lanes_join(aux, lanes, st0));
  return SI_OK;
}

// ----------------------------------------------------------------------------- Up/DownSample

struct ResamplePlan {
  int B, C, F, Hi, Wi, Ho, Wo, mode, TN, ncol;
  int64_t Pi, Po, slice_len, Mi_max;
  int lanes;
  size_t lane_stride, off_a, off_w, weights_bytes, total_bytes;
};

static si_status make_resample_plan(const si_tensor5* x, int32_t kind, int64_t slice_len, ResamplePlan* p) {
  if (!x) return SI_ERR_NULL;
  if (x->dtype != SI_BF16) return SI_ERR_DTYPE;
  if (kind != SI_RESAMPLE_DOWN && kind != SI_RESAMPLE_UP) return SI_ERR_ARG;
  if (x->B < 1 || x->C < 1 || x->F < 1 || x->H < 1 || x->W < 1) return SI_ERR_SHAPE;
  if (x->C % 32 || x->C > 8192 || x->B > 65535 || x->F > 65535 || x->H > 4096 || x->W > 4096) return SI_ERR_SHAPE;
  if (slice_len < 1) return SI_ERR_SLICE;
  p->B = (int)x->B; p->C = (int)x->C; p->F = (int)x->F; p->Hi = (int)x->H; p->Wi = (int)x->W;
  p->mode = kind == SI_RESAMPLE_DOWN ? kConvStride2 : kConvNearestUp;
  p->Ho = kind == SI_RESAMPLE_DOWN ? (p->Hi + 1) / 2 : 2 * p->Hi;
  p->Wo = kind == SI_RESAMPLE_DOWN ? (p->Wi + 1) / 2 : 2 * p->Wi;
  p->Pi = (int64_t)p->Hi * p->Wi;
  p->Po = (int64_t)p->Ho * p->Wo;
  if ((double)p->B * p->C * p->F * (double)(p->Pi > p->Po ? p->Pi : p->Po) >= 1099511627776.0) return SI_ERR_SHAPE;
  p->slice_len = slice_len < x->F ? slice_len : x->F;
  p->Mi_max = (int64_t)p->B * p->slice_len * p->Pi;
  if ((double)p->Mi_max * p->C * 2.0 + 4096.0 >= 4294967296.0) return SI_ERR_SHAPE;  // 32-bit operand offsets
  if ((int64_t)p->B * p->slice_len * p->Po >= (1LL << 31) / 16) return SI_ERR_SHAPE;
  const int64_t n_slices = (p->F + p->slice_len - 1) / p->slice_len;
  p->lanes = n_slices >= 8 ? 2 : 1;
  conv_column_tiles(p->C, ((int64_t)p->B * p->slice_len * p->Po + 127) / 128 * p->lanes, &p->TN, &p->ncol);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  p->off_a = take(kActZeroBytes + (size_t)((p->Mi_max + 31) / 32 * 32) * p->C * 2);
  p->lane_stride = off - p->off_a;
  if (p->lanes == 2) take(p->lane_stride);
  const size_t act_end = off;
  p->off_w = take((size_t)p->ncol * 9 * (p->C / 32) * 2 * p->TN * 1024);
  p->weights_bytes = off - act_end;
  p->total_bytes = off;
  return SI_OK;
}

static si_status run_resample(const ResamplePlan& p, const si_tensor5* x, const void* w_conv, const void* b_conv, si_tensor5* out,
                              char* ws, hipStream_t st0) {
  const bf16* X = static_cast<const bf16*>(x->ptr);
  bf16* OUT = static_cast<bf16*>(out->ptr);
  unsigned short* wf = reinterpret_cast<unsigned short*>(ws + p.off_w);
  const int C = p.C;
  {
    StageScope scope("pack_weights", st0);
    const int64_t elems = (int64_t)p.ncol * 9 * (C / 32) * 2 * p.TN * 512;
    unsigned* z0 = reinterpret_cast<unsigned*>(ws + p.off_a);
    pack_conv_kernel<false><<<(unsigned)((elems + 255) / 256), 256, 0, st0>>>(static_cast<const bf16*>(w_conv), wf, C, C, p.TN,
                                                                             p.ncol, z0, p.lanes, (int64_t)p.lane_stride);
    SI_CHECK_LAUNCH();
  }
  AuxStream* aux = nullptr;
  const int lanes = g_timing ? 1 : p.lanes;
  if (lanes == 2) {
    SI_TRY(aux_stream(&aux));
    SI_TRY(lanes_fork(aux, lanes, st0));
  }
  int widx = 0;
  for (int64_t f0 = 0; f0 < p.F; f0 += p.slice_len, ++widx) {
    const int lane_id = lanes == 2 ? widx & 1 : 0;
    hipStream_t st = lane_id ? aux->s[0] : st0;
    unsigned short* a = reinterpret_cast<unsigned short*>(ws + p.off_a + (size_t)lane_id * p.lane_stride);
    const int Fw = (int)((f0 + p.slice_len <= p.F) ? p.slice_len : p.F - f0);
    Window win_in{p.B, C, p.F, p.Pi, (int)f0, Fw, 0, (int)p.Pi, 1};
    Window win_out{p.B, C, p.F, p.Po, (int)f0, Fw, 0, (int)p.Po, 1};
    {
      StageScope scope("slice_in", st);
      dim3 grid((unsigned)((p.Pi + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)(p.B * Fw));
      window_to_tokens_silu_kernel<true><<<grid, 256, 0, st>>>(X, nullptr, nullptr, nullptr, a, win_in);
      SI_CHECK_LAUNCH();
    }
    EpiStoreRows epi{OUT, static_cast<const bf16*>(b_conv), win_out};
    SI_TRY(launch_conv3x3<false>(p.mode == kConvStride2 ? "conv_down" : "conv_up", a, wf, (int64_t)p.B * Fw * p.Po, C, p.TN,
                                 p.ncol, p.Ho, p.Wo, p.Hi, p.Wi, p.mode, epi, st));
  }
  if (lanes == 2) SI_TRY(lanes_join(aux, lanes, st0));
  return SI_OK;
}

}  // namespace si

extern "C" {

size_t si_resample_workspace_bytes(const si_tensor5* x, int32_t kind, int64_t slice_len) {
  si::ResamplePlan p;
  if (si::make_resample_plan(x, kind, slice_len, &p) != SI_OK) return 0;
  return p.total_bytes;
}

si_status si_resample_forward(const si_tensor5* x, int32_t kind, const void* w_conv, const void* b_conv, si_tensor5* out,
                              int64_t slice_len, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !out) return SI_ERR_NULL;
  si::ResamplePlan p;
  si_status s = si::make_resample_plan(x, kind, slice_len, &p);
  if (s != SI_OK) return s;
  if (out->dtype != x->dtype) return SI_ERR_DTYPE;
  if (out->B != x->B || out->C != x->C || out->F != x->F || out->H != p.Ho || out->W != p.Wo) return SI_ERR_SHAPE;
  if (!x->ptr || !out->ptr || !workspace || !w_conv) return SI_ERR_NULL;
  const void* all[] = {x->ptr, out->ptr, w_conv, b_conv};
  for (const void* q : all)
    if (q && !si::aligned16(q)) return SI_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SI_ERR_ALIGN;
  if (workspace_bytes < p.total_bytes) return SI_ERR_WORKSPACE;
  const size_t xbytes = (size_t)p.B * p.C * p.F * (size_t)p.Pi * 2, obytes = (size_t)p.B * p.C * p.F * (size_t)p.Po * 2;
  if (si::ranges_overlap(x->ptr, xbytes, out->ptr, obytes)) return SI_ERR_ARG;
  if (si::ranges_overlap(workspace, p.total_bytes, out->ptr, obytes) ||
      si::ranges_overlap(workspace, p.total_bytes, x->ptr, xbytes))
    return SI_ERR_ARG;
  return si::run_resample(p, x, w_conv, b_conv, out, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

size_t si_resblock_workspace_bytes(const si_tensor5* x, const si_resblock_weights* w, int64_t slice_len) {
  si::ResPlan p;
  if (si::make_res_plan(x, w, slice_len, &p) != SI_OK) return 0;
  return p.total_bytes;
}

size_t si_resblock_live_activation_bytes(const si_tensor5* x, const si_resblock_weights* w, int64_t slice_len) {
  si::ResPlan p;
  if (si::make_res_plan(x, w, slice_len, &p) != SI_OK) return 0;
  return p.total_bytes - p.weights_bytes;
}

si_status si_resblock_forward(const si_tensor5* x, const si_resblock_weights* w, const void* temb, si_tensor5* out,
                              int64_t slice_len, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !w || !out) return SI_ERR_NULL;
  si::ResPlan p;
  si_status s = si::make_res_plan(x, w, slice_len, &p);
  if (s != SI_OK) return s;
  if (out->dtype != x->dtype) return SI_ERR_DTYPE;
  if (out->B != x->B || out->C != p.Co || out->F != x->F || out->H != x->H || out->W != x->W) return SI_ERR_SHAPE;
  if (!x->ptr || !out->ptr || !workspace || !w->w_conv1 || !w->w_conv2) return SI_ERR_NULL;
  if (p.Kt > 0 && (!temb || !w->w_temb)) return SI_ERR_NULL;
  if (p.Co != p.C && !w->w_skip) return SI_ERR_NULL;
  const void* all[] = {x->ptr, out->ptr, temb, w->gn1_g, w->gn1_b, w->w_conv1, w->b_conv1, w->w_temb, w->b_temb,
                       w->gn2_g, w->gn2_b, w->w_conv2, w->b_conv2, w->w_skip, w->b_skip};
  for (const void* q : all)
    if (q && !si::aligned16(q)) return SI_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SI_ERR_ALIGN;
  if (workspace_bytes < p.total_bytes) return SI_ERR_WORKSPACE;
  const size_t xbytes = (size_t)p.B * p.C * p.F * (size_t)p.P * 2, obytes = (size_t)p.B * p.Co * p.F * (size_t)p.P * 2;
  if (si::ranges_overlap(x->ptr, xbytes, out->ptr, obytes)) return SI_ERR_ARG;
  if (si::ranges_overlap(workspace, p.total_bytes, out->ptr, obytes) ||
      si::ranges_overlap(workspace, p.total_bytes, x->ptr, xbytes))
    return SI_ERR_ARG;
  return si::run_resblock(p, x, w, temb, out, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

}  // extern "C"
