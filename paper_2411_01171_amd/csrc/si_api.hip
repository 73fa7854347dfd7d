// C ABI of the Streamlined-Inference hot path (see include/si.h): argument
// validation, workspace layout, the host slice loop (Feature Slicer windows,
// Sec. 4.1; one operator group per window, Sec. 4.2.1) and kernel launches.
#include "../../include/si.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "k_attn.h"
#include "k_cosine.h"
#include "k_fused.h"
#include "k_fused_attn.h"
#include "k_fused_block.h"
#include "k_fused_pre.h"
#include "k_attn_mfma.h"
#include "k_conv.h"
#include "k_gemm.h"
#include "k_norm.h"
#include "si_common.h"

namespace si {

// ----------------------------------------------------------------------------- stage timing

struct StageEvent {
  int stage;
  hipEvent_t a, b;
};
static bool g_timing = false;
static std::vector<std::string> g_stage_names;
static std::vector<StageEvent> g_events;

static int stage_id(const char* name) {
  for (size_t i = 0; i < g_stage_names.size(); ++i)
    if (g_stage_names[i] == name) return (int)i;
  g_stage_names.emplace_back(name);
  return (int)g_stage_names.size() - 1;
}

struct StageScope {
  hipStream_t st;
  StageEvent ev;
  bool on;
  StageScope(const char* name, hipStream_t s) : st(s), on(g_timing) {
    if (!on) return;
    ev.stage = stage_id(name);
    if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(ev.a, st);
  }
  ~StageScope() {
    if (!on) return;
    (void)hipEventRecord(ev.b, st);
    g_events.push_back(ev);
  }
};

// ----------------------------------------------------------------------------- plan

constexpr int kMaxLanes = 3;  // windows in flight at most (measured: a fourth window in flight gains nothing at 25 slices
                              // and 7 % at 16, where it would take the live bytes past a quarter of the unsliced run's)

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Column tiles of the ring kernel used as a GEMM on windows of up to Mmax tokens (`lanes` of them in
// flight) x N columns over K: the widest tile (5, 4, 2 or 1 blocks of 32 columns) that pads N by at
// most a tenth and still gives enough workgroups of 128 tokens, else the narrowest such tile.
// Enough (measured): for long k loops (K > 512) 330 workgroups over the windows in flight, and never
// the 32-column tile if a wider one fits (64-column tiles beat both the wider and the narrower ones
// whenever the wider ones leave fewer: cfg5's N = 1280 at 2048 tokens, cfg3's N = 640 at 2048 to
// 8192 tokens); for short k loops 400 in the launch itself.  Weight packing and launch use the same
// arguments.
struct RingDims {
  int64_t Mmax;
  int lanes;
};
struct RingShape {
  int tn, ncol;
};
static RingShape ring_shape(RingDims d, int N, int K) {
  // q/k/v of one window in flight at the deep levels (N = 3 K = 3840 on 2048 tokens): 128-column tiles make
  // 480 workgroups, two for nearly every CU, where 160-column tiles make 384 (measured 34.0 -> 31.5 us)
  if (d.lanes == 1 && K > 512 && N == 3 * K && N % 128 == 0) {
    const int64_t wg = (d.Mmax + 127) / 128 * (N / 128);
    if (wg > 448 && wg <= 512) return RingShape{4, N / 128};
  }
  // one window in flight and a projection whose 64-column tiles would give some CUs two workgroups and most of
  // them one (N = 1280 on 2048 tokens: 320): 96-column tiles make it one workgroup for nearly every CU (224)
  if (d.lanes == 1 && K > 512 && N % 32 == 0) {
    const int64_t rows128 = (d.Mmax + 127) / 128;
    const int nc3 = (N + 95) / 96;
    if (rows128 * ((N + 63) / 64) > 256 && rows128 * nc3 <= 256 && rows128 * nc3 > 160 && (int64_t)nc3 * 96 * 10 <= (int64_t)N * 11)
      return RingShape{3, nc3};
  }
  const int64_t rows = (d.Mmax + 127) / 128 * (K > 512 ? d.lanes : 1);
  const int min_wg = K > 512 ? 330 : 400;
  RingShape best{1, (N + 31) / 32};
  bool found = false;
  for (int tn : {5, 4, 2, 1}) {
    const int nc = (N + 32 * tn - 1) / (32 * tn);
    if ((int64_t)nc * tn * 32 * 10 > (int64_t)N * 11) continue;  // too much padding
    if (tn == 1 && K > 512 && found) break;
    best = RingShape{tn, nc};
    found = true;
    if (rows * nc >= min_wg) break;
  }
  return best;
}

struct Plan {
  int kind, dtype, esize;
  int B, C, F, H, W, G, heads, d, D;
  int64_t P;
  int Mc, Cc;    // context tokens / width (spatial)
  int axis;
  int64_t extent, slice_len;
  int64_t Mmax;  // tokens of the largest window
  bool pe;
  int fused_nb;     // > 0: register-resident FFN half with D = 32*fused_nb
  bool fused_attn;  // register-resident attention half as well (temporal blocks)
  bool attn_split;  // fused_attn, cut behind the attention: the FFN half runs as a kernel of its own on dense
                    // token tiles (F leaves many of a wavefront's 32 columns empty in the one-kernel form)
  bool post_fused;  // spatial: everything behind the self-attention (its out-projection, LN2, query projection,
                    // attention over the context, FFN half) in one register-resident kernel
  bool attn_mfma;   // matrix-core attention kernel for the staged spatial path (bf16, head dimension 64)
  bool ring;        // staged bf16 GEMMs run on the fragment-order ring kernel (operands in fragment order)
  int lanes;        // slices in flight (many small slices: 2 or 3, each on a stream of its own)
  size_t lane_stride;  // bytes between two lanes' slice intermediates
  int Mcp;          // context tokens rounded up to a multiple of 8 (transposed value copy)
  // workspace offsets (bytes)
  size_t off_stats, off_rehash, off_pe, off_ctxkv, off_ctxvt, off_vt;
  size_t off_w_in, off_wqkv, off_wo, off_wq2, off_wkv2, off_wo2, off_w1, off_w2, off_w_out;
  size_t off_a, off_h, off_big, off_ffn_stream, off_attn_stream, off_pre_stream;
  size_t weights_bytes, total_bytes;
};

// sub-chunks of context fragments per batch entry in the post-attention kernel's stream
static int post_ctx_sub(const Plan& p) { return (p.D / 64) * kCrossOps / (2 * p.fused_nb); }

static si_status make_plan(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, int32_t axis,
                           int64_t slice_len, Plan* p) {
  if (!x || !w) return SI_ERR_NULL;
  if (x->dtype != SI_F32 && x->dtype != SI_BF16) return SI_ERR_DTYPE;
  if (w->kind != SI_BLOCK_TEMPORAL && w->kind != SI_BLOCK_SPATIAL) return SI_ERR_ARG;
  if (x->B < 1 || x->C < 1 || x->F < 1 || x->H < 1 || x->W < 1) return SI_ERR_SHAPE;
  if (w->heads < 1 || w->dim_head < 8 || w->dim_head > 128 || w->dim_head % 8) return SI_ERR_SHAPE;
  if (w->gn_groups < 1 || x->C % w->gn_groups || x->C % 8) return SI_ERR_SHAPE;
  const int64_t D = (int64_t)w->heads * w->dim_head;
  if (D > 2048 || x->C > 8192) return SI_ERR_SHAPE;
  const int64_t P = x->H * x->W;
  if (x->B > 65535 || x->F > 65535 || P > (1 << 24)) return SI_ERR_SHAPE;
  if ((double)x->B * x->C * x->F * (double)P >= 1099511627776.0) return SI_ERR_SHAPE;
  if ((int64_t)(x->C / w->gn_groups) * P >= (1LL << 31)) return SI_ERR_SHAPE;
  if (!(w->gn_eps >= 0.f) || !(w->ln_eps >= 0.f)) return SI_ERR_ARG;
  p->kind = w->kind;
  p->dtype = x->dtype;
  p->esize = x->dtype == SI_F32 ? 4 : 2;
  p->B = (int)x->B; p->C = (int)x->C; p->F = (int)x->F; p->H = (int)x->H; p->W = (int)x->W;
  p->P = P; p->G = w->gn_groups; p->heads = w->heads; p->d = w->dim_head; p->D = (int)D;
  p->Mc = 0; p->Cc = 0;
  if (w->kind == SI_BLOCK_SPATIAL) {
    if (!ctx) return SI_ERR_NULL;
    if (ctx->dtype != x->dtype) return SI_ERR_DTYPE;
    if (ctx->B != x->B || ctx->M < 1 || ctx->M > 65535 || ctx->Cc < 1 || ctx->Cc > 65536) return SI_ERR_SHAPE;
    if (ctx->Cc % 8) return SI_ERR_SHAPE;
    if (w->add_sin_pe) return SI_ERR_ARG;
    p->Mc = (int)ctx->M;
    p->Cc = (int)ctx->Cc;
  }
  p->pe = w->kind == SI_BLOCK_TEMPORAL && w->add_sin_pe != 0;
  if (axis != SI_AXIS_F && axis != SI_AXIS_HW) return SI_ERR_SLICE;
  if ((axis == SI_AXIS_F) != (w->kind == SI_BLOCK_SPATIAL)) return SI_ERR_SLICE;
  if (slice_len < 1) return SI_ERR_SLICE;
  p->axis = axis;
  p->extent = axis == SI_AXIS_F ? x->F : P;
  p->slice_len = slice_len < p->extent ? slice_len : p->extent;
  p->Mmax = axis == SI_AXIS_F ? (int64_t)x->B * p->slice_len * P : (int64_t)x->B * x->F * p->slice_len;
  if (p->Mmax >= (1LL << 31) / 16) return SI_ERR_SHAPE;

  const size_t es = (size_t)p->esize;
  const size_t C = (size_t)p->C, Dz = (size_t)D;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  // slice-independent activation-derived items
  p->off_stats = take((size_t)p->B * p->F * p->G * 2 * sizeof(float));
  p->off_ctxkv = take((size_t)p->B * p->Mc * 2 * Dz * es);
  p->attn_mfma = p->dtype == SI_BF16 && p->kind == SI_BLOCK_SPATIAL && p->d == 64 && P % 8 == 0;
  p->Mcp = (p->Mc + 7) / 8 * 8;
  p->off_ctxvt = take(p->attn_mfma ? (size_t)p->B * Dz * p->Mcp * es : 0);
  // which path: register-resident kernels need bf16, C == D = 64 or 320 (instantiated widths)
  p->fused_nb = 0;
  p->fused_attn = false;
  p->attn_split = false;
  if (p->dtype == SI_BF16 && p->C == p->D && (D == 64 || D == 320)) {
    p->fused_nb = (int)(D / 32);
    const int tp = p->F <= 32 ? 32 / p->F : 0;
    const bool dh_ok = (D == 320 && (p->d == 40 || p->d == 64)) || (D == 64 && p->d == 32);
    // a workgroup (up to 128 consecutive positions) keeps the statistics of two batch entries: every
    // window, the shorter last one included, must be at least that long unless B <= 2
    const int64_t last_len = p->extent % p->slice_len ? p->extent % p->slice_len : p->slice_len;
    p->fused_attn = p->kind == SI_BLOCK_TEMPORAL && tp >= 1 && dh_ok && (int64_t)p->F * p->G <= kAttnMaxStats &&
                    (p->B <= 2 || last_len >= 128);
    // columns of a wavefront that hold no token in the one-kernel form: 32 - floor(32 / F) * F
    p->attn_split = p->fused_attn && (32 - tp * p->F) * 100 >= 15 * 32;
  }
  // a workgroup's 128 tokens share one context (P % 128 == 0: frames are whole workgroups), heads of 64
  // channels (two 32-channel blocks), at most kCrossTiles key tiles
  p->post_fused = p->fused_nb == 10 && p->kind == SI_BLOCK_SPATIAL && p->attn_mfma && p->d == 64 && P % 128 == 0 &&
                  p->Mc <= 32 * kCrossTiles;
  // Ring GEMMs: 16-bit storage, every contraction length a multiple of the 32-wide k-tile, operand
  // buffers addressable with 32-bit byte offsets.
  p->ring = p->dtype == SI_BF16 && p->C % 32 == 0 && D % 32 == 0 &&
            (double)p->Mmax * (double)(4 * D > p->C ? 4 * D : p->C) * 2.0 + 4096.0 < 4294967296.0;
  // one slice's intermediates
  if (p->fused_attn) {  // one kernel per window: only the parked residual stream (128 rows per workgroup)
    const int64_t npos = 4 * (32 / p->F);
    const int64_t wgs = ((int64_t)p->B * p->slice_len + npos - 1) / npos;
    // attn_split: the attention output and the residual stream as token rows (+ 4 KiB that idle lanes write to)
    const size_t Mt = (size_t)((p->Mmax + 127) / 128 * 128);  // whole 128-token tiles
    p->off_a = take(p->attn_split ? Mt * Dz * es : 0);
    p->off_h = take(p->attn_split ? Mt * Dz * sizeof(float) + 4096 : (size_t)wgs * 128 * Dz * sizeof(float));
    p->off_big = take(0);
  } else {
    // fragment-order operand buffers carry a 256-byte head and whole 32-token blocks
    const size_t pad = p->ring ? kActZeroBytes : 0, Mp = p->ring ? (size_t)((p->Mmax + 31) / 32 * 32) : (size_t)p->Mmax;
    p->off_a = take(pad + Mp * (C > Dz ? C : Dz) * es);
    p->off_h = take((size_t)p->Mmax * Dz * sizeof(float));
    p->off_big = take(pad + Mp * 4 * Dz * es);
  }
  p->off_vt = take(p->attn_mfma ? (size_t)p->Mmax * Dz * es : 0);  // values of the window, keys contiguous
  // Cross-slice pipelining (Sec. 4.2.2): with many small slices the kernels of one slice leave CUs
  // idle (under-filled grids, partial last rounds), so several windows run at a time, each on a
  // stream and with intermediates of its own: as many as keep the window intermediates in flight
  // within a quarter of what the unsliced run needs for them (one per four slices, at most
  // kMaxLanes).  The slice-independent items (statistics, frame table, context keys / values) come
  // on top in either case.
  const int64_t n_slices = (p->extent + p->slice_len - 1) / p->slice_len;
  p->lanes = (int)(n_slices / 4 < 1 ? 1 : n_slices / 4 > kMaxLanes ? kMaxLanes : n_slices / 4);
  p->lane_stride = off - p->off_a;
  for (int l = 1; l < p->lanes; ++l) take(p->lane_stride);
  // Similarity partials of the fused statistics + rehash pass (3 doubles per block), then {cos, decision}:
  // written and read back before the first window starts, so they lie in the first window's intermediates
  // when those are large enough.
  const size_t rehash_bytes = (size_t)p->B * p->F * p->G * 3 * sizeof(double) + 16;
  p->off_rehash = rehash_bytes <= p->lane_stride ? p->off_a : take(rehash_bytes);
  const size_t act_end = off;
  // frame position table (a function of F and D only: written with the weight re-layout)
  p->off_pe = take(p->pe ? (size_t)p->F * Dz * sizeof(float) : 0);
  // re-laid-out weights ([N, K]; fragment streams pad N to whole column tiles)
  auto wbytes = [&](size_t N, size_t K) {
    if (!p->ring) return N * K * es;
    const RingShape rs = ring_shape(RingDims{p->Mmax, p->lanes}, (int)N, (int)K);
    return (size_t)rs.ncol * rs.tn * 32 * K * es;
  };
  p->off_w_in = take(wbytes(Dz, C));
  p->off_wqkv = take(wbytes(3 * Dz, Dz));
  p->off_wo = take(wbytes(Dz, Dz));
  const bool sp = p->kind == SI_BLOCK_SPATIAL;
  p->off_wq2 = take(sp ? wbytes(Dz, Dz) : 0);
  p->off_wkv2 = take(sp ? 2 * Dz * (size_t)p->Cc * es : 0);
  p->off_wo2 = take(sp ? wbytes(Dz, Dz) : 0);
  p->off_w1 = take(wbytes(8 * Dz, Dz));
  p->off_w2 = take(wbytes(Dz, 4 * Dz));
  p->off_w_out = take(wbytes(C, Dz));
  // post_fused: + W_o and W_q2 blocks and, per batch entry, the context fragments (24 per head)
  const int ffn_sub = 14 * p->fused_nb + (p->post_fused ? 2 * p->fused_nb + post_ctx_sub(*p) * p->B : 0);
  p->off_ffn_stream = take(p->fused_nb && (!p->fused_attn || p->attn_split) ? (size_t)stream_bytes(ffn_sub, 2 * p->fused_nb) : 0);
  p->off_attn_stream = take(p->fused_attn ? (size_t)stream_bytes((p->attn_split ? 4 : 18) * p->fused_nb, 2 * p->fused_nb) : 0);
  // post_fused: the kernel in front of the self-attention takes W_in, W_q, W_k, W_v as a stream of its own
  p->off_pre_stream = take(p->post_fused ? (size_t)stream_bytes(4 * p->fused_nb, 2 * p->fused_nb) : 0);
  p->weights_bytes = off - act_end;
  p->total_bytes = off;
  return SI_OK;
}

// ----------------------------------------------------------------------------- launches

#define SI_CHECK_LAUNCH()                         \
  do {                                            \
    if (hipGetLastError() != hipSuccess) return SI_ERR_HIP; \
  } while (0)

template <typename T, class Epi, int BK, bool F16>
static void launch_gemm_bf16(const T* A, int64_t lda, const T* Wp, int64_t M, int N, int K, Epi epi, hipStream_t st) {
  // small problems (a slice of a few thousand tokens times a D-wide matrix) get 64 x 64 tiles:
  // four times the workgroups, so that every CU has work
  if (((M + 127) / 128) * ((N + 127) / 128) < 256) {
    dim3 grid((unsigned)((M + 63) / 64), (unsigned)((N + 63) / 64));
    gemm_bf16_kernel<64, 64, 2, 2, Epi, BK, F16><<<grid, 256, 0, st>>>(A, lda, Wp, M, N, K, epi);
  } else if (N % 128 == 0) {
    dim3 grid((unsigned)((M + 127) / 128), (unsigned)(N / 128));
    gemm_bf16_kernel<128, 128, 2, 2, Epi, BK, F16><<<grid, 256, 0, st>>>(A, lda, Wp, M, N, K, epi);
  } else {
    dim3 grid((unsigned)((M + 127) / 128), (unsigned)((N + 63) / 64));
    gemm_bf16_kernel<128, 64, 4, 1, Epi, BK, F16><<<grid, 256, 0, st>>>(A, lda, Wp, M, N, K, epi);
  }
}

// F16: both 16-bit operands hold fp16 values (proj_in / proj_out of the bf16 staged path).
template <typename T, bool F16 = false, class Epi>
static si_status launch_gemm(const char* stage, const T* A, int64_t lda, const T* Wp, int64_t M, int N, int K, Epi epi,
                             hipStream_t st) {
  if (M <= 0) return SI_OK;
  StageScope scope(stage, st);
  if constexpr (sizeof(T) == 4) {
    dim3 grid((unsigned)((M + 63) / 64), (unsigned)((N + 63) / 64));
    gemm_f32_kernel<Epi><<<grid, 256, 0, st>>>(A, lda, Wp, M, N, K, epi);
  } else {
    // short contractions (K = 320: five 64-wide tiles) run better with 32-wide k tiles: half the LDS,
    // twice the workgroups per CU to hide the pipeline's fill and drain
    if (K <= 512) launch_gemm_bf16<T, Epi, 32, F16>(A, lda, Wp, M, N, K, epi, st);
    else launch_gemm_bf16<T, Epi, 64, F16>(A, lda, Wp, M, N, K, epi, st);
  }
  SI_CHECK_LAUNCH();
  return SI_OK;
}

// batch: collect eligible matrices instead of launching; flush_pack launches them all at once
template <typename T>
static si_status launch_pack(const T* src, T* dst, int K, int ld_src, int rows, int col0, int interleave, hipStream_t st,
                             int ld_dst = 0, bool to_f16 = false, int frag_tn = 0, int frag_row0 = 0, PackBatch* batch = nullptr) {
  if (!ld_dst) ld_dst = K;
  if (sizeof(T) == 2 && col0 == 0 && K % 8 == 0 && ld_dst % 8 == 0 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
    if (batch && batch->n < kPackBatchMax) {
      const int bx = (rows + 63) / 64, by = (K + 63) / 64;
      batch->job[batch->n++] = PackJob{reinterpret_cast<const unsigned short*>(src), reinterpret_cast<unsigned short*>(dst), K, ld_src,
                                       rows, interleave, ld_dst, to_f16 ? 1 : 0, frag_tn, frag_row0, K, batch->blocks, bx};
      batch->blocks += bx * by;
      return SI_OK;
    }
    dim3 grid((unsigned)((rows + 63) / 64), (unsigned)((K + 63) / 64));
    pack_transpose16_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const unsigned short*>(src), reinterpret_cast<unsigned short*>(dst),
                                                  K, ld_src, rows, interleave, ld_dst, to_f16 ? 1 : 0, frag_tn, frag_row0, K);
  } else {
    dim3 grid((unsigned)((rows + 31) / 32), (unsigned)((K + 31) / 32));
    pack_transpose_kernel<T><<<grid, 256, 0, st>>>(src, dst, K, ld_src, rows, col0, interleave, ld_dst, to_f16 ? 1 : 0, frag_tn,
                                                   frag_row0, K);
  }
  SI_CHECK_LAUNCH();
  return SI_OK;
}

// One [K, rows] parameter matrix into rows [row0, row0 + rows) of the packed [N_total, K] weight at
// `base`: k-contiguous rows, or (as_ring) the ring kernel's fragment stream for problems of up to
// Mmax tokens.  f16: 16-bit values are stored as fp16.
template <typename T>
static si_status pack_weight(const T* src, T* base, int K, int ld_src, int rows, int interleave, int N_total, int row0,
                             bool as_ring, RingDims Mmax, bool f16, hipStream_t st, PackBatch* batch = nullptr) {
  if (as_ring)
    return launch_pack<T>(src, base, K, ld_src, rows, 0, interleave, st, K, f16, ring_shape(Mmax, N_total, K).tn, row0, batch);
  return launch_pack<T>(src, base + (size_t)row0 * K, K, ld_src, rows, 0, interleave, st, K, f16, 0, 0, batch);
}
static si_status flush_pack(const PackBatch& batch, hipStream_t st) {
  if (batch.n == 0) return SI_OK;
  pack_transpose16_batch_kernel<<<(unsigned)batch.blocks, 256, 0, st>>>(batch);
  SI_CHECK_LAUNCH();
  return SI_OK;
}

// The ring kernel (k_conv.h) as a GEMM: M tokens are M one-pixel images, one tap; act is a
// fragment-order operand buffer (K channels per token), wf the fragment stream packed by
// pack_weight for (Mmax, N).  Same epilogue contract as gemm_bf16_kernel.
template <bool F16, class Epi>
static si_status launch_gemm_ring(const char* stage, const void* act, const void* wf, int64_t M, RingDims Mmax, int N, int K,
                                  Epi epi, hipStream_t st) {
  if (M <= 0) return SI_OK;
  StageScope scope(stage, st);
  const RingShape rs = ring_shape(Mmax, N, K);
  // 256-token row tiles for the largest problems only: 400 workgroups over the windows in flight
  // (measured: cfg3's ff1 with three windows in flight gains 4 % per step although one launch
  // alone is slower, 31 -> 43 us)
  constexpr int kBigMin = 400;
  const int64_t rows2 = (M + 255) / 256;
  const bool big = rs.tn >= 4 && rows2 * rs.ncol * Mmax.lanes >= kBigMin;
  ConvArgs a{static_cast<const char*>(act), static_cast<const char*>(wf), M, K, N, 1, 1, rs.ncol,
             (int)((big ? rows2 : (M + 127) / 128) * rs.ncol), 1, 1, kConvSame, 1,
             M < N ? 1 : 0};  // the smaller operand is the one every XCD streams
  const unsigned grid = (unsigned)((a.ntiles + 7) / 8 * 8);
  // Narrow tiles (64 or 32 columns: the N = D projections and ff2) run wavefront-specialised: their
  // launches have one or two workgroups per CU, too few to hide a workgroup's load issue behind
  // another's MFMAs (measured per step: cfg3 1.68 -> 1.59 ms, cfg5 spatial 1.33 -> 1.29 ms, cfg5 temporal
  // 1.12 -> 1.08 ms; the 160-column tiles of q/k/v and ff1 lose with it: two such workgroups no longer
  // fit a CU's registers).
  if (!big && rs.tn <= 3) {
    // ff2 of one window in flight (K = 4 N): 256-token row tiles, one workgroup per CU at most, move fewer
    // ring bytes per MFMA than 320 tiles of 128 tokens on 256 CUs (measured 52.7 -> 50.9 us at cfg5)
    if (rs.tn == 2 && M >= 1024 && Mmax.lanes == 1 && K >= 4 * N && rows2 * rs.ncol <= 256) {
      a.ntiles = (int)(rows2 * rs.ncol);
      ring_mma_kernel<2, 2, 4, F16, Epi, true><<<(unsigned)((a.ntiles + 7) / 8 * 8), 512, 0, st>>>(a, epi);
    } else if (rs.tn == 3) ring_mma_kernel<1, 3, 4, F16, Epi, true><<<grid, 512, 0, st>>>(a, epi);
    else if (rs.tn == 2) ring_mma_kernel<1, 2, 4, F16, Epi, true><<<grid, 512, 0, st>>>(a, epi);
    else ring_mma_kernel<1, 1, 6, F16, Epi, true><<<grid, 512, 0, st>>>(a, epi);
    SI_CHECK_LAUNCH();
    return SI_OK;
  }
  switch (rs.tn * 2 + (big ? 1 : 0)) {
    case 11: ring_mma_kernel<2, 5, 3, F16, Epi><<<grid, 256, 0, st>>>(a, epi); break;
    case 10: ring_mma_kernel<1, 5, 4, F16, Epi><<<grid, 256, 0, st>>>(a, epi); break;
    case 9: ring_mma_kernel<2, 4, 3, F16, Epi><<<grid, 256, 0, st>>>(a, epi); break;
    case 8: ring_mma_kernel<1, 4, 4, F16, Epi><<<grid, 256, 0, st>>>(a, epi); break;
    default: return SI_ERR_ARG;  // ring_shape only gives tiles of 1, 2, 3, 4 or 5 column blocks
  }
  SI_CHECK_LAUNCH();
  return SI_OK;
}

// as_ring: A is a fragment-order buffer and Wp a fragment stream -> ring kernel; else rows of lda.
template <typename T, bool F16, class Epi>
static si_status launch_gemm_sel(const char* stage, bool as_ring, const T* A, int64_t lda, const T* Wp, int64_t M, RingDims Mmax,
                                 int N, int K, Epi epi, hipStream_t st) {
  if constexpr (sizeof(T) == 2) {
    if (as_ring) return launch_gemm_ring<F16>(stage, A, Wp, M, Mmax, N, K, epi, st);
  }
  return launch_gemm<T, F16>(stage, A, lda, Wp, M, N, K, epi, st);
}

template <typename T>
static si_status launch_attention(const char* stage, const AttnArgs& a, hipStream_t st) {
  if (a.S <= 0 || a.Nq <= 0) return SI_OK;
  StageScope scope(stage, st);
  if constexpr (sizeof(T) == 2) {
    // self-attention over a short sequence (temporal blocks): one wavefront per (sequence, head)
    const bool rows16 = a.ldq % 8 == 0 && a.ldk % 8 == 0 && a.ldv % 8 == 0 && a.ldo % 8 == 0 && aligned16(a.q) && aligned16(a.k) &&
                        aligned16(a.v) && aligned16(a.o);
    if (a.d == 64 && a.Nq == a.Nk && a.Nk <= 32 && rows16) {
      attn_short_kernel<64><<<(unsigned)(((int64_t)a.S * a.heads + 3) / 4), 256, 0, st>>>(a);
      SI_CHECK_LAUNCH();
      return SI_OK;
    }
  }
  constexpr int QB = 4;
  dim3 grid((unsigned)((a.Nq + 4 * QB - 1) / (4 * QB)), (unsigned)a.heads, (unsigned)a.S);
  attn_valu_kernel<T, QB><<<grid, 256, 0, st>>>(a);
  SI_CHECK_LAUNCH();
  return SI_OK;
}

// Matrix-core attention (bf16, head dimension 64): v is first copied with keys contiguous.
static si_status launch_attention_mfma(const char* stage, const bf16* q, int64_t ldq, const bf16* k, int64_t ldk,
                                       const bf16* vt, bf16* o, int64_t ldo, int S, int Nq, int Nk, int Nkp, int heads,
                                       int kv_div, hipStream_t st, int o_frag = 0) {
  if (S <= 0 || Nq <= 0) return SI_OK;
  StageScope scope(stage, st);
  AttnMfmaArgs a;
  a.q = q; a.ldq = ldq; a.k = k; a.ldk = ldk; a.vt = vt; a.o = o; a.ldo = ldo;
  a.Nq = Nq; a.Nk = Nk; a.Nkp = Nkp; a.heads = heads; a.kv_div = kv_div;
  a.o_frag = o_frag;
  a.ksplit = 1; a.o2 = nullptr; a.ml = nullptr; a.tiles32 = 0;
  // 8 wavefronts share the key / value stages when that still leaves several workgroups for every CU
  const int64_t wg8 = (int64_t)((Nq + 255) / 256) * heads * S;
  if (wg8 >= 1024) {
    a.nqt = (Nq + 255) / 256;
    a.ntiles = a.nqt * heads * S;
    attn_mfma_kernel<8><<<(unsigned)((a.ntiles + 7) / 8 * 8), 512, 0, st>>>(a);
  } else {
    a.nqt = (Nq + 127) / 128;
    a.ntiles = a.nqt * heads * S;
    attn_mfma_kernel<4><<<(unsigned)((a.ntiles + 7) / 8 * 8), 256, 0, st>>>(a);
  }
  SI_CHECK_LAUNCH();
  return SI_OK;
}
static si_status launch_transpose_v(const char* stage, const bf16* src, int64_t ld, int col0, bf16* dst, int S, int N, int Nkp,
                                    int D, hipStream_t st) {
  if (S <= 0 || N <= 0) return SI_OK;
  StageScope scope(stage, st);
  dim3 grid((unsigned)((Nkp + 31) / 32), (unsigned)((D + 31) / 32), (unsigned)S);
  transpose_v_kernel<<<grid, 256, 0, st>>>(src, ld, col0, dst, N, Nkp, D);
  SI_CHECK_LAUNCH();
  return SI_OK;
}

template <typename T>
static si_status launch_layer_norm(const char* stage, const float* h, T* a, int64_t M, int D, const void* g, const void* b,
                                   float eps, const float* pe, int Pw, int Fw, int f0, hipStream_t st, bool frag = false) {
  StageScope scope(stage, st);
  const unsigned blocks = (unsigned)((M + 3) / 4);
  if (frag && sizeof(T) == 2) {
    if constexpr (sizeof(T) == 2) {
      const unsigned wgs = (unsigned)((M + 7) / 8);
      const bf16 *gp = static_cast<const bf16*>(g), *bp = static_cast<const bf16*>(b);
      bf16* ap = reinterpret_cast<bf16*>(a);
      // large windows at the widths of the five configurations run on the eight-rows-per-wavefront
      // kernel; with few rows one wavefront per row keeps more of the chip busy (measured at 2048
      // rows: 9 us against 15 at D = 640, 12 against 25 at D = 1280; at 18432 rows, D = 320: 21 against 14),
      // eight rows per workgroup so that the stores are whole 128-byte pieces (2048 rows: 9.3 -> 7.9 us
      // at D = 640, 12.2 -> 9.6 at D = 1280)
      switch (M >= 8192 ? D : 0) {
        case 320: layer_norm_frag_kernel<10><<<wgs, 64, 0, st>>>(h, ap, M, gp, bp, eps, pe, Pw, Fw, f0); break;
        case 640: layer_norm_frag_kernel<20><<<wgs, 64, 0, st>>>(h, ap, M, gp, bp, eps, pe, Pw, Fw, f0); break;
        case 1280: layer_norm_frag_kernel<40><<<wgs, 64, 0, st>>>(h, ap, M, gp, bp, eps, pe, Pw, Fw, f0); break;
        default:
          if (D % 8 == 0 && D <= 2048 && (!g || aligned16(g)) && (!b || aligned16(b)))
            layer_norm_rows8_kernel<<<wgs, 512, 0, st>>>(h, ap, M, D, gp, bp, eps, pe, Pw, Fw, f0);
          else
            layer_norm_kernel<T, sizeof(T) == 2><<<blocks, 256, 0, st>>>(h, a, M, D, static_cast<const T*>(g), static_cast<const T*>(b),
                                                                         eps, pe, Pw, Fw, f0);
      }
    }
  }
  else
    layer_norm_kernel<T><<<blocks, 256, 0, st>>>(h, a, M, D, static_cast<const T*>(g), static_cast<const T*>(b), eps, pe, Pw, Fw, f0);
  SI_CHECK_LAUNCH();
  return SI_OK;
}

#define SI_TRY(expr)                  \
  do {                                \
    si_status st__ = (expr);          \
    if (st__ != SI_OK) return st__;   \
  } while (0)

// Fragment stream of the register-resident kernels (bf16 only) and the frame table, one launch.
template <int NB>
static si_status pack_fused_streams(const Plan& p, const si_block_weights* w, char* ws, float* pe, hipStream_t st) {
  const int D = p.D;
  auto cB = [](const void* q) { return static_cast<const bf16*>(q); };
  const bool spatial = p.kind == SI_BLOCK_SPATIAL;
  StreamDesc sd;
  int n = 0;
  if (p.attn_split) {  // the attention half's blocks as a stream of their own (with the frame table)
    StreamDesc ad;
    int k = 0;
    const int gw = lcm_int(p.d, 32), nbg = gw / 32, ng = D / gw;
    for (int nb = 0; nb < NB; ++nb) ad.b[k++] = BlockDesc{cB(w->w_in), D, 32 * nb, 0};
    for (int gi = 0; gi < ng; ++gi) {
      const void* mats[3] = {w->wq, w->wk, w->wv};
      for (int kind = 0; kind < 3; ++kind)
        for (int blk = 0; blk < nbg; ++blk) ad.b[k++] = BlockDesc{cB(mats[kind]), D, gi * gw + 32 * blk, 0};
    }
    ad.n_pre = k; ad.n_post = 0; ad.n_ffn = 0; ad.extra_sub = 0;
    ad.w1 = ad.w2 = nullptr; ad.pe = pe; ad.F = p.F;
    const int pe_wgs = pe ? (p.F * D + 255) / 256 : 0;
    pack_stream_kernel<NB><<<(k * 2 * NB + 3) / 4 + pe_wgs, 256, 0, st>>>(ad, reinterpret_cast<u32x4_t*>(ws + p.off_attn_stream));
    SI_CHECK_LAUNCH();
    pe = nullptr;  // written
  } else if (p.fused_attn) {  // attention half: W_in blocks, then per head group q, k, v blocks
    const int gw = lcm_int(p.d, 32), nbg = gw / 32, ng = D / gw;
    for (int nb = 0; nb < NB; ++nb) sd.b[n++] = BlockDesc{cB(w->w_in), D, 32 * nb, 0};
    for (int gi = 0; gi < ng; ++gi) {
      const void* mats[3] = {w->wq, w->wk, w->wv};
      for (int kind = 0; kind < 3; ++kind)
        for (int blk = 0; blk < nbg; ++blk) sd.b[n++] = BlockDesc{cB(mats[kind]), D, gi * gw + 32 * blk, 0};
    }
  }
  if (p.post_fused) {  // self-attention out-projection and the query projection of the context attention
    for (int nb = 0; nb < NB; ++nb) sd.b[n++] = BlockDesc{cB(w->wo), D, 32 * nb, 0};
    for (int nb = 0; nb < NB; ++nb) sd.b[n++] = BlockDesc{cB(w->wq2), D, 32 * nb, 0};
  }
  // FFN half: out-projection of the last attention, FFN, proj_out
  for (int nb = 0; nb < NB; ++nb) sd.b[n++] = BlockDesc{cB(spatial ? w->wo2 : w->wo), D, 32 * nb, 0};
  sd.n_pre = n;
  for (int nb = 0; nb < NB; ++nb) sd.b[n++] = BlockDesc{cB(w->w_out), p.C, 32 * nb, 0};
  sd.n_post = NB;
  sd.w1 = cB(w->w1); sd.w2 = cB(w->w2);
  sd.pe = pe; sd.F = p.F;
  sd.extra_sub = p.post_fused ? post_ctx_sub(p) * p.B : 0;
  sd.n_ffn = 12 * NB;
  const int total = sd.n_pre + 12 * NB + sd.n_post;
  u32x4_t* stream = reinterpret_cast<u32x4_t*>(ws + (p.fused_attn && !p.attn_split ? p.off_attn_stream : p.off_ffn_stream));
  const int frag_wgs = (total * 2 * NB + 3) / 4, pe_wgs = pe ? (p.F * D + 255) / 256 : 0;
  pack_stream_kernel<NB><<<frag_wgs + pe_wgs, 256, 0, st>>>(sd, stream);
  SI_CHECK_LAUNCH();
  if (p.post_fused) {  // the stream of the kernel in front of the self-attention: W_in (as fp16), W_q, W_k, W_v
    StreamDesc pd;
    int k = 0;
    for (int nb = 0; nb < NB; ++nb) pd.b[k++] = BlockDesc{cB(w->w_in), D, 32 * nb, 1};
    const void* mats[3] = {w->wq, w->wk, w->wv};
    for (int kind = 0; kind < 3; ++kind)
      for (int nb = 0; nb < NB; ++nb) pd.b[k++] = BlockDesc{cB(mats[kind]), D, 32 * nb, 0};
    pd.n_pre = k; pd.n_post = 0; pd.n_ffn = 0; pd.extra_sub = 0;
    pd.w1 = pd.w2 = nullptr; pd.pe = nullptr; pd.F = 0;
    pack_stream_kernel<NB><<<(k * 2 * NB + 3) / 4, 256, 0, st>>>(pd, reinterpret_cast<u32x4_t*>(ws + p.off_pre_stream));
    SI_CHECK_LAUNCH();
  }
  return SI_OK;
}

// Auxiliary streams and fork / join events for windows in flight, one set per device, created on
// first use (default priority) and kept for the life of the process.  Calls that overlap on one
// device share them and must not run concurrently from several host threads.
struct AuxStream {
  hipStream_t s[kMaxLanes - 1] = {};   // lane l >= 1 runs on s[l - 1]; lane 0 on the caller's stream
  hipEvent_t fork = nullptr, join[kMaxLanes - 1] = {};
};
static si_status aux_stream(AuxStream** out) {
  static AuxStream per_device[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SI_ERR_HIP;
  AuxStream& a = per_device[dev];
  if (!a.fork) {
    for (int l = 0; l < kMaxLanes - 1; ++l) {
      if (hipStreamCreateWithFlags(&a.s[l], hipStreamNonBlocking) != hipSuccess) return SI_ERR_HIP;
      if (hipEventCreateWithFlags(&a.join[l], hipEventDisableTiming) != hipSuccess) return SI_ERR_HIP;
    }
    if (hipEventCreateWithFlags(&a.fork, hipEventDisableTiming) != hipSuccess) return SI_ERR_HIP;
  }
  *out = &a;
  return SI_OK;
}
// fork: the other lanes start after what the caller's stream has enqueued so far
static si_status lanes_fork(AuxStream* aux, int lanes, hipStream_t st_main) {
  if (hipEventRecord(aux->fork, st_main) != hipSuccess) return SI_ERR_HIP;
  for (int l = 1; l < lanes; ++l)
    if (hipStreamWaitEvent(aux->s[l - 1], aux->fork, 0) != hipSuccess) return SI_ERR_HIP;
  return SI_OK;
}
// join: the caller's stream continues after all lanes
static si_status lanes_join(AuxStream* aux, int lanes, hipStream_t st_main) {
  for (int l = 1; l < lanes; ++l)
    if (hipEventRecord(aux->join[l - 1], aux->s[l - 1]) != hipSuccess || hipStreamWaitEvent(st_main, aux->join[l - 1], 0) != hipSuccess)
      return SI_ERR_HIP;
  return SI_OK;
}

// GroupNorm statistics of the whole feature; with `key` the same pass also leaves the similarity
// partials of x against key (one triple per block) at off_rehash.
template <typename T>
static si_status launch_gn_stats(const Plan& p, const T* X, const T* key, float eps, char* ws, hipStream_t st) {
  StageScope scope(key ? "gn_stats_cosine" : "gn_stats", st);
  constexpr int VEC = 16 / sizeof(T);
  float* stats = reinterpret_cast<float*>(ws + p.off_stats);
  double* partial = reinterpret_cast<double*>(ws + p.off_rehash);
  const unsigned blocks = (unsigned)(p.B * p.F * p.G);
  if (p.P % VEC == 0) {
    if (key) gn_stats_kernel<T, VEC, true><<<blocks, 256, 0, st>>>(X, stats, p.C, p.F, p.P, p.G, eps, key, partial);
    else gn_stats_kernel<T, VEC><<<blocks, 256, 0, st>>>(X, stats, p.C, p.F, p.P, p.G, eps);
  } else {
    if (key) gn_stats_kernel<T, 1, true><<<blocks, 256, 0, st>>>(X, stats, p.C, p.F, p.P, p.G, eps, key, partial);
    else gn_stats_kernel<T, 1><<<blocks, 256, 0, st>>>(X, stats, p.C, p.F, p.P, p.G, eps);
  }
  SI_CHECK_LAUNCH();
  return SI_OK;
}

template <typename T>
static si_status run_block(const Plan& p, const si_tensor5* x, const si_block_weights* w, const si_context* ctx,
                           si_tensor5* out, char* ws, hipStream_t st, bool stats_done = false, bool packed = false) {
  const T* X = static_cast<const T*>(x->ptr);
  T* OUT = static_cast<T*>(out->ptr);
  float* stats = reinterpret_cast<float*>(ws + p.off_stats);
  float* pe = p.pe ? reinterpret_cast<float*>(ws + p.off_pe) : nullptr;
  T* ctxkv = reinterpret_cast<T*>(ws + p.off_ctxkv);
  T* a = reinterpret_cast<T*>(ws + p.off_a);
  float* h = reinterpret_cast<float*>(ws + p.off_h);
  T* big = reinterpret_cast<T*>(ws + p.off_big);
  T* w_in = reinterpret_cast<T*>(ws + p.off_w_in);
  T* wqkv = reinterpret_cast<T*>(ws + p.off_wqkv);
  T* wo = reinterpret_cast<T*>(ws + p.off_wo);
  T* wq2 = reinterpret_cast<T*>(ws + p.off_wq2);
  T* wkv2 = reinterpret_cast<T*>(ws + p.off_wkv2);
  T* wo2 = reinterpret_cast<T*>(ws + p.off_wo2);
  T* w1 = reinterpret_cast<T*>(ws + p.off_w1);
  T* w2 = reinterpret_cast<T*>(ws + p.off_w2);
  T* w_out = reinterpret_cast<T*>(ws + p.off_w_out);
  const int C = p.C, D = p.D;
  const bool spatial = p.kind == SI_BLOCK_SPATIAL;
  const bool fused_ffn = p.fused_nb > 0, fused_attn = p.fused_attn;
  constexpr bool kF16 = sizeof(T) == 2;  // proj_in / proj_out run on fp16 operands for 16-bit storage
  // operand buffers in fragment order + ring kernel; the attention outputs too where the matrix-core
  // attention kernel writes them and a staged GEMM (not the FFN-half kernel) reads them
  const bool ring = p.ring;
  const bool self_frag = ring && p.attn_mfma && !p.post_fused, cross_frag = ring && p.attn_mfma && !fused_ffn;
  const RingDims Mx{p.Mmax, p.lanes};
  auto cT = [](const void* q) { return static_cast<const T*>(q); };

  // ---- once per call: weight re-layout, frame embedding table (skipped when the caller vouches that
  // the workspace still holds them), GroupNorm statistics, context K/V
  if (!packed) {
    StageScope scope("pack_weights", st);
    PackBatch pb;
    pb.n = 0;
    pb.blocks = 0;
    PackBatch* const pbp = &pb;
    if (!fused_attn && !p.post_fused) {
      SI_TRY(pack_weight<T>(cT(w->w_in), w_in, C, D, D, 0, D, 0, ring, Mx, kF16, st, pbp));
      SI_TRY(pack_weight<T>(cT(w->wq), wqkv, D, D, D, 0, 3 * D, 0, ring, Mx, false, st, pbp));
      SI_TRY(pack_weight<T>(cT(w->wk), wqkv, D, D, D, 0, 3 * D, D, ring, Mx, false, st, pbp));
      SI_TRY(pack_weight<T>(cT(w->wv), wqkv, D, D, D, 0, 3 * D, 2 * D, ring, Mx, false, st, pbp));
      if ((spatial || !fused_ffn) && !p.post_fused)
        SI_TRY(pack_weight<T>(cT(w->wo), wo, D, D, D, 0, D, 0, self_frag, Mx, false, st, pbp));
    }
    if (spatial) {
      if (!p.post_fused) SI_TRY(pack_weight<T>(cT(w->wq2), wq2, D, D, D, 0, D, 0, ring, Mx, false, st, pbp));
      SI_TRY(launch_pack<T>(cT(w->wk2), wkv2, p.Cc, D, D, 0, 0, st, 0, false, 0, 0, pbp));
      SI_TRY(launch_pack<T>(cT(w->wv2), wkv2 + (size_t)D * p.Cc, p.Cc, D, D, 0, 0, st, 0, false, 0, 0, pbp));
      if (!fused_ffn) SI_TRY(pack_weight<T>(cT(w->wo2), wo2, D, D, D, 0, D, 0, cross_frag, Mx, false, st, pbp));
    }
    if (!fused_ffn) {
      SI_TRY(pack_weight<T>(cT(w->w_out), w_out, D, C, C, 0, C, 0, ring, Mx, kF16, st, pbp));
      SI_TRY(pack_weight<T>(cT(w->w1), w1, D, 8 * D, 8 * D, 4 * D, 8 * D, 0, ring, Mx, false, st, pbp));
      SI_TRY(pack_weight<T>(cT(w->w2), w2, 4 * D, D, D, 0, D, 0, ring, Mx, false, st, pbp));
    } else if constexpr (sizeof(T) == 2) {
      if (p.fused_nb == 2) SI_TRY(pack_fused_streams<2>(p, w, ws, pe, st));
      else SI_TRY(pack_fused_streams<10>(p, w, ws, pe, st));
    }
    SI_TRY(flush_pack(pb, st));
    if (pe && !(fused_ffn && sizeof(T) == 2)) {
      pe_table_kernel<<<(p.F * D + 255) / 256, 256, 0, st>>>(pe, p.F, D);
      SI_CHECK_LAUNCH();
    }
  }
  if (!stats_done) SI_TRY(launch_gn_stats<T>(p, X, nullptr, w->gn_eps, ws, st));
  if (spatial) {
    EpiStore<T> epi{ctxkv, (int64_t)2 * D, nullptr};
    SI_TRY(launch_gemm<T>("ctx_kv", cT(ctx->ptr), (int64_t)p.Cc, wkv2, (int64_t)p.B * p.Mc, 2 * D, p.Cc, epi, st));
    if constexpr (sizeof(T) == 2) {
      if (p.post_fused) {  // the context as fragments behind the post-attention kernel's weight stream
        StageScope scope("ctx_frags", st);
        const int n_main = 16 * p.fused_nb, per_b = post_ctx_sub(p);
        const int64_t pitch = stream_pitch_u4(n_main + per_b * p.B);
        const unsigned wgs = (unsigned)((p.B * per_b * 2 * p.fused_nb + 3) / 4);
        pack_ctx_stream_kernel<10><<<wgs, 256, 0, st>>>(ctxkv, p.B, p.Mc, reinterpret_cast<u32x4_t*>(ws + p.off_ffn_stream), pitch,
                                                        n_main);
        SI_CHECK_LAUNCH();
      } else if (p.attn_mfma)
        SI_TRY(launch_transpose_v("ctx_vt", ctxkv, (int64_t)2 * D, D, reinterpret_cast<bf16*>(ws + p.off_ctxvt), p.B, p.Mc, p.Mcp, D, st));
    }
  }

  // ---- Feature Slicer windows; one operator group per window (Eq. 1)
  const float scale = 1.0f / sqrtf((float)p.d);
  // the matrix-core attention kernel exponentiates in base 2 and takes its queries pre-scaled: the
  // projections that feed it fold softmax scale * log2(e) into q before q's one rounding
  const float qscale2 = scale * 1.4426950408889634f;
  hipStream_t const st_main = st;
  T* const a_base = a;
  float* const h_base = h;
  T* const big_base = big;
  AuxStream* aux = nullptr;
  // per-stage timing wants each kernel alone on the GPU: one window at a time while it is enabled
  const int lanes = g_timing ? 1 : p.lanes;
  if (lanes >= 2) {  // fork: the other lanes start after the once-per-call work above
    SI_TRY(aux_stream(&aux));
    SI_TRY(lanes_fork(aux, lanes, st_main));
  }
  for (int64_t s0 = 0; s0 < p.extent; s0 += p.slice_len) {
    const int64_t s1 = s0 + p.slice_len < p.extent ? s0 + p.slice_len : p.extent;
    // this slice's lane: stream and intermediates (the names below shadow the first lane's)
    const int lane_id = (int)((s0 / p.slice_len) % lanes);
    const size_t lane_off = (size_t)lane_id * p.lane_stride;
    hipStream_t st = lane_id == 0 ? st_main : aux->s[lane_id - 1];
    T* a = reinterpret_cast<T*>(reinterpret_cast<char*>(a_base) + lane_off);
    float* h = reinterpret_cast<float*>(reinterpret_cast<char*>(h_base) + lane_off);
    T* big = reinterpret_cast<T*>(reinterpret_cast<char*>(big_base) + lane_off);
    char* const vt_lane = ws + p.off_vt + lane_off;
    (void)vt_lane;
    Window win;
    win.B = p.B; win.C = C; win.F = p.F; win.P = p.P; win.G = p.G;
    if (p.axis == SI_AXIS_F) {
      win.f0 = (int)s0; win.Fw = (int)(s1 - s0); win.p0 = 0; win.Pw = (int)p.P;
    } else {
      win.f0 = 0; win.Fw = p.F; win.p0 = s0; win.Pw = (int)(s1 - s0);
    }
    const int64_t M = (int64_t)p.B * win.Fw * win.Pw;

    if constexpr (sizeof(T) == 2) {
      if (fused_attn) {  // the whole operator group of the window in one kernel (attn_split: up to the attention)
        StageScope scope(p.attn_split ? "attn_half_fused" : "temporal_block_fused", st);
        TemporalBlockArgs ta;
        ta.x = X; ta.out = OUT; ta.stats = stats;
        ta.gn_g = cT(w->gn_g); ta.gn_b = cT(w->gn_b); ta.b_in = cT(w->b_in);
        ta.ln1_g = cT(w->ln1_g); ta.ln1_b = cT(w->ln1_b); ta.b_o = cT(w->bo);
        ta.ln3_g = cT(w->ln3_g); ta.ln3_b = cT(w->ln3_b); ta.b1 = cT(w->b1); ta.b2 = cT(w->b2); ta.b_out = cT(w->b_out);
        ta.pe = pe; ta.stream = reinterpret_cast<const u32x4_t*>(ws + p.off_attn_stream);
        ta.hpark = h; ta.o_rows = a; ta.ln_eps = w->ln_eps; ta.scale = scale; ta.win = win;
        const int npos = 4 * (32 / p.F);
        const unsigned blocks = (unsigned)(((int64_t)p.B * win.Pw + npos - 1) / npos);
        if (p.attn_split) {
          if (p.fused_nb == 2) temporal_block_kernel<2, 32, true><<<blocks, 256, 0, st>>>(ta);
          else if (p.d == 40) temporal_block_kernel<10, 40, true><<<blocks, 256, 0, st>>>(ta);
          else temporal_block_kernel<10, 64, true><<<blocks, 256, 0, st>>>(ta);
        } else {
          if (p.fused_nb == 2) temporal_block_kernel<2, 32><<<blocks, 256, 0, st>>>(ta);
          else if (p.d == 40) temporal_block_kernel<10, 40><<<blocks, 256, 0, st>>>(ta);
          else temporal_block_kernel<10, 64><<<blocks, 256, 0, st>>>(ta);
        }
        SI_CHECK_LAUNCH();
        if (!p.attn_split) continue;
      }
    }
    int ksplit = 1;
    if constexpr (sizeof(T) == 2) {
      if (p.post_fused) {  // slice-in, proj_in, LN1, q / k / v in one kernel, then the self-attention
        {
          StageScope scope("pre_attn_fused", st);
          SpatialPreArgs pa;
          pa.x = X; pa.stats = stats;
          pa.gn_g = cT(w->gn_g); pa.gn_b = cT(w->gn_b); pa.b_in = cT(w->b_in); pa.ln_g = cT(w->ln1_g); pa.ln_b = cT(w->ln1_b);
          pa.stream = reinterpret_cast<const u32x4_t*>(ws + p.off_pre_stream);
          pa.h = h; pa.qf = reinterpret_cast<u32x4_t*>(big); pa.kvf = reinterpret_cast<u32x4_t*>(big + M * D);
          pa.M = M; pa.ln_eps = w->ln_eps; pa.qscale = qscale2; pa.win = win;
          spatial_pre_kernel<10><<<(unsigned)(M / 128), 256, 0, st>>>(pa);
          SI_CHECK_LAUNCH();
        }
        {  // operands and output as fragments (q: M*D values at big, k / v^T stage blocks behind them)
          StageScope scope("self_attn", st);
          AttnMfmaArgs aa;
          aa.q = big; aa.ldq = 0; aa.k = big + M * D; aa.ldk = 0; aa.vt = nullptr; aa.o = a; aa.ldo = 0;
          aa.Nq = aa.Nk = aa.Nkp = win.Pw; aa.heads = p.heads; aa.kv_div = 1; aa.o_frag = 0;
          aa.nqt = win.Pw / 128;
          // two key halves per query tile when one workgroup per tile would leave the last round of
          // workgroups (2 per CU) less than half full; the halves' statistics live in the (otherwise
          // unused) transposed-value buffer, the second half's output behind q, k, v
          const int64_t wgs1 = (int64_t)aa.nqt * p.heads * p.B * win.Fw;
          aa.ksplit = (win.Pw % 256 == 0 && wgs1 > 512 && wgs1 % 512 > 0 && wgs1 % 512 <= 256) ? 2 : 1;
          ksplit = aa.ksplit;
          aa.o2 = big + 3 * M * D;
          aa.ml = reinterpret_cast<float2*>(vt_lane);
          aa.tiles32 = M / 32;
          aa.ntiles = (int)(wgs1 * aa.ksplit);
          attn_mfma_kernel<4, true><<<(unsigned)((aa.ntiles + 7) / 8 * 8), 256, 0, st>>>(aa);
          SI_CHECK_LAUNCH();
        }
      }
    }
    if (!fused_attn && !p.post_fused) {
      {  // slice-in: window -> GroupNorm -> token rows
        StageScope scope("slice_in", st);
        dim3 grid((unsigned)((win.Pw + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)(p.B * win.Fw));
        if constexpr (sizeof(T) == 2) {
          if (ring) window_to_tokens_f16_kernel<true><<<grid, 256, 0, st>>>(X, stats, cT(w->gn_g), cT(w->gn_b), a, win);
          else window_to_tokens_f16_kernel<false><<<grid, 256, 0, st>>>(X, stats, cT(w->gn_g), cT(w->gn_b), a, win);
        } else
          window_to_tokens_kernel<T><<<grid, 256, 0, st>>>(X, stats, cT(w->gn_g), cT(w->gn_b), a, win);
        SI_CHECK_LAUNCH();
      }
      {
        EpiResidual<T> epi{h, (int64_t)D, cT(w->b_in), 0, nullptr};
        SI_TRY((launch_gemm_sel<T, kF16>("proj_in", ring, a, (int64_t)C, w_in, M, Mx, D, C, epi, st)));
      }
      SI_TRY(launch_layer_norm<T>("ln1", h, a, M, D, w->ln1_g, w->ln1_b, w->ln_eps, pe, win.Pw, win.Fw, win.f0, st, ring));
      bool self_done = false;
      if constexpr (sizeof(T) == 2) {
        if (p.attn_mfma) {  // spatial: sequence (b, f) = rows (b*Fw + f)*Pw + i; the projection writes V transposed
          bf16* vt = reinterpret_cast<bf16*>(vt_lane);
          EpiStoreQKVt epi{big, (int64_t)3 * D, vt, D, win.Pw, qscale2};
          SI_TRY((launch_gemm_sel<T, false>("qkv", ring, a, (int64_t)D, wqkv, M, Mx, 3 * D, D, epi, st)));
          SI_TRY(launch_attention_mfma("self_attn", big, (int64_t)3 * D, big + D, (int64_t)3 * D, vt, a, (int64_t)D, p.B * win.Fw,
                                       win.Pw, win.Pw, win.Pw, p.heads, 1, st, self_frag ? D : 0));
          self_done = true;
        }
      }
      if (!self_done) {
        {
          EpiStore<T> epi{big, (int64_t)3 * D, nullptr};
          SI_TRY((launch_gemm_sel<T, false>("qkv", ring, a, (int64_t)D, wqkv, M, Mx, 3 * D, D, epi, st)));
        }
        AttnArgs at;
        at.q = big; at.k = big + D; at.v = big + 2 * D; at.o = a;
        at.ldq = at.ldk = at.ldv = (int64_t)3 * D; at.ldo = D;
        at.heads = p.heads; at.d = p.d; at.scale = scale;
        if (spatial) {
          at.S = p.B * win.Fw; at.Nq = at.Nk = win.Pw;
          at.qmap = SeqMap{1, (int64_t)win.Pw, 0, 1};
        } else {
          at.S = p.B * win.Pw; at.Nq = at.Nk = p.F;
          at.qmap = SeqMap{win.Pw, (int64_t)p.F * win.Pw, 1, (int64_t)win.Pw};
        }
        at.kmap = at.qmap;
        SI_TRY(launch_attention<T>("self_attn", at, st));
      }
      if ((spatial || !fused_ffn) && !p.post_fused) {  // otherwise the FFN-half kernel applies W_o itself
        EpiResidual<T> epi{h, (int64_t)D, cT(w->bo), 1, nullptr};
        SI_TRY((launch_gemm_sel<T, false>("attn_out", self_frag, a, (int64_t)D, wo, M, Mx, D, D, epi, st)));
      }
      if (spatial && !p.post_fused) {
        SI_TRY(launch_layer_norm<T>("ln2", h, a, M, D, w->ln2_g, w->ln2_b, w->ln_eps, nullptr, win.Pw, win.Fw, win.f0, st, ring));
        {
          EpiStore<T> epi{big, (int64_t)D, nullptr, p.attn_mfma ? qscale2 : 1.f};
          SI_TRY((launch_gemm_sel<T, false>("q2", ring, a, (int64_t)D, wq2, M, Mx, D, D, epi, st)));
        }
        bool cross_done = false;
        if constexpr (sizeof(T) == 2) {
          if (p.attn_mfma) {  // keys / values: the context rows of the batch entry, shared by its frames
            SI_TRY(launch_attention_mfma("cross_attn", big, (int64_t)D, ctxkv, (int64_t)2 * D,
                                         reinterpret_cast<const bf16*>(ws + p.off_ctxvt), a, (int64_t)D, p.B * win.Fw, win.Pw,
                                         p.Mc, p.Mcp, p.heads, win.Fw, st, cross_frag ? D : 0));
            cross_done = true;
          }
        }
        if (!cross_done) {
          AttnArgs at;
          at.q = big; at.k = ctxkv; at.v = ctxkv + D; at.o = a;
          at.ldq = D; at.ldk = at.ldv = (int64_t)2 * D; at.ldo = D;
          at.heads = p.heads; at.d = p.d; at.scale = scale;
          at.S = p.B * win.Fw; at.Nq = win.Pw; at.Nk = p.Mc;
          at.qmap = SeqMap{1, (int64_t)win.Pw, 0, 1};
          at.kmap = SeqMap{win.Fw, (int64_t)p.Mc, 0, 1};
          SI_TRY(launch_attention<T>("cross_attn", at, st));
        }
        if (!fused_ffn) {
          EpiResidual<T> epi{h, (int64_t)D, cT(w->bo2), 1, nullptr};
          SI_TRY((launch_gemm_sel<T, false>("cross_out", cross_frag, a, (int64_t)D, wo2, M, Mx, D, D, epi, st)));
        }
      }
    }
    if constexpr (sizeof(T) == 2) {
      if (fused_ffn) {  // h += a W_o + b_o, LN3, GEGLU FFN, proj_out, residual, slice-out
        StageScope scope(p.post_fused ? "post_attn_fused" : "ffn_half_fused", st);
        FfnHalfArgs fa;
        fa.h = h; fa.o = a; fa.M = M; fa.stream = reinterpret_cast<const u32x4_t*>(ws + p.off_ffn_stream);
        fa.b_o = cT(spatial && !p.post_fused ? w->bo2 : w->bo);
        fa.ln_g = cT(w->ln3_g); fa.ln_b = cT(w->ln3_b); fa.b1 = cT(w->b1); fa.b2 = cT(w->b2); fa.b_out = cT(w->b_out);
        fa.ln_eps = w->ln_eps; fa.x = X; fa.out = OUT; fa.win = win;
        fa.ln2_g = fa.ln2_b = fa.b_o2 = nullptr;
        fa.pitch = 0; fa.ctx_sub0 = 0; fa.Mc = 0; fa.tokens_per_batch = 128; fa.qscale = 0.f; fa.h_tiled = 0;
        fa.o2 = nullptr; fa.ml = nullptr; fa.tiles32 = 0;
        if (p.attn_split) fa.h_tiled = 1;  // the attention half leaves tile-order residual rows and operand fragments
        const unsigned blocks = (unsigned)((M + 127) / 128);
        if (p.post_fused) {  // `a` holds the self-attention output; the kernel goes on from there
          fa.ln2_g = cT(w->ln2_g); fa.ln2_b = cT(w->ln2_b); fa.b_o2 = cT(w->bo2);
          fa.ctx_sub0 = 16 * p.fused_nb;
          fa.pitch = stream_pitch_u4(fa.ctx_sub0 + post_ctx_sub(p) * p.B);
          fa.Mc = p.Mc; fa.tokens_per_batch = (int)(win.Fw * win.Pw); fa.qscale = qscale2;
          fa.h_tiled = 1;
          if (ksplit == 2) {
            fa.o2 = big + 3 * M * D; fa.ml = reinterpret_cast<const float2*>(vt_lane); fa.tiles32 = M / 32;
          }
          ffn_half_kernel<10, true><<<blocks, 256, 0, st>>>(fa);
        } else if (p.fused_nb == 2) ffn_half_kernel<2><<<blocks, 256, 0, st>>>(fa);
        else ffn_half_kernel<10><<<blocks, 256, 0, st>>>(fa);
        SI_CHECK_LAUNCH();
        continue;
      }
    }
    SI_TRY(launch_layer_norm<T>("ln3", h, a, M, D, w->ln3_g, w->ln3_b, w->ln_eps, nullptr, win.Pw, win.Fw, win.f0, st, ring));
    bool ffn_done = false;
    if constexpr (sizeof(T) == 2) {
      if (ring) {  // GEGLU output, the final residual stream and the slice-out all in / from fragment order
        EpiGeglu<T, true> e1{big, (int64_t)4 * D, cT(w->b1), 4 * D};
        SI_TRY((launch_gemm_ring<false>("ff1_geglu", a, w1, M, Mx, 8 * D, D, e1, st)));
        EpiResidual<T, true> e2{h, (int64_t)D, cT(w->b2), 1, a};  // also leaves the final h as fp16 in `a`
        SI_TRY((launch_gemm_ring<false>("ff2", big, w2, M, Mx, D, 4 * D, e2, st)));
        EpiSliceOutRows e3{X, OUT, cT(w->b_out), win};
        SI_TRY((launch_gemm_ring<true>("proj_out", a, w_out, M, Mx, C, D, e3, st)));
        ffn_done = true;
      }
    }
    if (!ffn_done) {
      {
        EpiGeglu<T> epi{big, (int64_t)4 * D, cT(w->b1), 4 * D};
        SI_TRY(launch_gemm<T>("ff1_geglu", a, (int64_t)D, w1, M, 8 * D, D, epi, st));
      }
      {
        EpiResidual<T> epi{h, (int64_t)D, cT(w->b2), 1, a};  // also leaves the final h as T in `a`
        SI_TRY(launch_gemm<T>("ff2", big, (int64_t)4 * D, w2, M, D, 4 * D, epi, st));
      }
      {
        EpiSliceOut<T> epi{X, OUT, cT(w->b_out), win};
        SI_TRY((launch_gemm<T, kF16>("proj_out", a, (int64_t)D, w_out, M, C, D, epi, st)));
      }
    }
  }
  if (lanes >= 2) SI_TRY(lanes_join(aux, lanes, st_main));
  return SI_OK;
}

// What the host can verify of a SI_FWD_WEIGHTS_PACKED promise: the last call that re-laid-out weights
// into this workspace (in this process, on this device) had the same plan -- every offset, tile choice
// and stream length follows from the fields hashed here -- and the same parameter pointers.  A small
// table of the most recent workspaces, shared by all callers and guarded by a mutex.
static uint64_t fnv1a(uint64_t h, const void* data, size_t n) {
  const unsigned char* b = static_cast<const unsigned char*>(data);
  for (size_t i = 0; i < n; ++i) h = (h ^ b[i]) * 1099511628211ull;
  return h;
}
static uint64_t pack_fingerprint(const Plan& p, const si_block_weights* w) {
  int dev = -1;
  (void)hipGetDevice(&dev);
  const int64_t f[] = {p.kind, p.dtype, p.B, p.C, p.F, p.H, p.W, p.G, p.heads, p.d, p.Mc, p.Cc, p.axis, p.extent, p.slice_len,
                       p.Mmax, p.pe, p.fused_nb, p.fused_attn, p.attn_split, p.post_fused, p.attn_mfma, p.ring, p.lanes, (int64_t)p.weights_bytes,
                       (int64_t)p.total_bytes, (int64_t)p.off_w_in, (int64_t)p.off_ffn_stream, (int64_t)p.off_attn_stream, dev};
  uint64_t h = fnv1a(14695981039346656037ull, f, sizeof(f));
  const void* q[] = {w->gn_g, w->gn_b, w->w_in, w->b_in, w->ln1_g, w->ln1_b, w->wq, w->wk, w->wv, w->wo, w->bo,
                     w->ln3_g, w->ln3_b, w->w1, w->b1, w->w2, w->b2, w->w_out, w->b_out};
  h = fnv1a(h, q, sizeof(q));
  if (p.kind == SI_BLOCK_SPATIAL) {
    const void* sp[] = {w->ln2_g, w->ln2_b, w->wq2, w->wk2, w->wv2, w->wo2, w->bo2};
    h = fnv1a(h, sp, sizeof(sp));
  }
  return h ? h : 1;
}
struct PackRecord {
  const void* ws;
  uint64_t fp;
};
static std::mutex g_pack_mutex;
static PackRecord g_pack_table[64];
static unsigned g_pack_next = 0;
static void pack_record(const void* ws, uint64_t fp) {
  std::lock_guard<std::mutex> lock(g_pack_mutex);
  for (PackRecord& r : g_pack_table)
    if (r.ws == ws) {
      r.fp = fp;
      return;
    }
  g_pack_table[g_pack_next++ % 64] = PackRecord{ws, fp};
}
static bool pack_matches(const void* ws, uint64_t fp) {
  std::lock_guard<std::mutex> lock(g_pack_mutex);
  for (const PackRecord& r : g_pack_table)
    if (r.ws == ws) return r.fp == fp;
  return false;
}

static bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + nb && b0 < a0 + na;
}

}  // namespace si

#include "si_resblock_api.h"

// ============================================================================= C ABI

extern "C" {

int32_t si_abi_version(void) { return 1; }

const char* si_status_str(int32_t s) {
  switch (s) {
    case SI_OK: return "ok";
    case SI_ERR_NULL: return "required pointer is NULL";
    case SI_ERR_SHAPE: return "inconsistent or unsupported shape";
    case SI_ERR_DTYPE: return "unknown or mismatching dtype";
    case SI_ERR_SLICE: return "illegal slice axis or length";
    case SI_ERR_ALIGN: return "misaligned device pointer";
    case SI_ERR_WORKSPACE: return "workspace too small";
    case SI_ERR_ARG: return "invalid argument";
    case SI_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

size_t si_workspace_bytes(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, int32_t axis,
                          int64_t slice_len) {
  si::Plan p;
  if (si::make_plan(x, w, ctx, axis, slice_len, &p) != SI_OK) return 0;
  return p.total_bytes;
}

size_t si_live_activation_bytes(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, int32_t axis,
                                int64_t slice_len) {
  si::Plan p;
  if (si::make_plan(x, w, ctx, axis, slice_len, &p) != SI_OK) return 0;
  return p.total_bytes - p.weights_bytes;
}

int32_t si_windows_in_flight(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, int32_t axis,
                             int64_t slice_len) {
  si::Plan p;
  if (si::make_plan(x, w, ctx, axis, slice_len, &p) != SI_OK) return 0;
  return p.lanes;
}

// Argument checks shared by the forward entry points; fills the plan.
static si_status check_forward(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, si_tensor5* out,
                               int32_t axis, int64_t slice_len, void* workspace, size_t workspace_bytes, si::Plan& p) {
  if (!x || !w || !out) return SI_ERR_NULL;
  si_status s = si::make_plan(x, w, ctx, axis, slice_len, &p);
  if (s != SI_OK) return s;
  if (out->dtype != x->dtype) return SI_ERR_DTYPE;
  if (out->B != x->B || out->C != x->C || out->F != x->F || out->H != x->H || out->W != x->W) return SI_ERR_SHAPE;
  if (!x->ptr || !out->ptr || !workspace) return SI_ERR_NULL;
  const void* req[] = {w->w_in, w->wq, w->wk, w->wv, w->wo, w->w1, w->w2, w->w_out};
  for (const void* q : req)
    if (!q) return SI_ERR_NULL;
  const bool spatial = w->kind == SI_BLOCK_SPATIAL;
  if (spatial) {
    if (!ctx->ptr || !w->wq2 || !w->wk2 || !w->wv2 || !w->wo2) return SI_ERR_NULL;
  }
  const void* all[] = {x->ptr, out->ptr, w->gn_g, w->gn_b, w->w_in, w->b_in, w->ln1_g, w->ln1_b, w->wq, w->wk, w->wv,
                       w->wo, w->bo, w->ln3_g, w->ln3_b, w->w1, w->b1, w->w2, w->b2, w->w_out, w->b_out};
  for (const void* q : all)
    if (q && !si::aligned16(q)) return SI_ERR_ALIGN;
  if (spatial) {
    const void* sp[] = {ctx->ptr, w->ln2_g, w->ln2_b, w->wq2, w->wk2, w->wv2, w->wo2, w->bo2};
    for (const void* q : sp)
      if (q && !si::aligned16(q)) return SI_ERR_ALIGN;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SI_ERR_ALIGN;
  if (workspace_bytes < p.total_bytes) return SI_ERR_WORKSPACE;
  const size_t xbytes = (size_t)p.B * p.C * p.F * (size_t)p.P * p.esize;
  if (si::ranges_overlap(x->ptr, xbytes, out->ptr, xbytes)) return SI_ERR_ARG;
  if (si::ranges_overlap(workspace, p.total_bytes, out->ptr, xbytes) ||
      si::ranges_overlap(workspace, p.total_bytes, x->ptr, xbytes))
    return SI_ERR_ARG;
  return SI_OK;
}

si_status si_block_forward_ex(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, si_tensor5* out,
                              int32_t axis, int64_t slice_len, void* workspace, size_t workspace_bytes, uint32_t flags,
                              void* stream) {
  if (flags & ~(uint32_t)SI_FWD_WEIGHTS_PACKED) return SI_ERR_ARG;
  si::Plan p;
  si_status s = check_forward(x, w, ctx, out, axis, slice_len, workspace, workspace_bytes, p);
  if (s != SI_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const bool packed = (flags & SI_FWD_WEIGHTS_PACKED) != 0;
  const uint64_t fp = si::pack_fingerprint(p, w);
  if (packed && !si::pack_matches(workspace, fp)) return SI_ERR_ARG;  // nothing enqueued
  if (!packed) si::pack_record(workspace, fp);
  if (p.dtype == SI_F32) return si::run_block<float>(p, x, w, ctx, out, ws, st, false, packed);
  return si::run_block<si::bf16>(p, x, w, ctx, out, ws, st, false, packed);
}

si_status si_block_forward(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, si_tensor5* out,
                           int32_t axis, int64_t slice_len, void* workspace, size_t workspace_bytes, void* stream) {
  return si_block_forward_ex(x, w, ctx, out, axis, slice_len, workspace, workspace_bytes, 0u, stream);
}

si_status si_block_forward_rehash(const si_tensor5* x, const si_block_weights* w, const si_context* ctx, si_tensor5* out,
                                  int32_t axis, int64_t slice_len, void* workspace, size_t workspace_bytes,
                                  si_rehash_cache* cache, float gamma, void* stream, double* cos_host,
                                  int32_t* reused_host) {
  si::Plan p;
  si_status s = check_forward(x, w, ctx, out, axis, slice_len, workspace, workspace_bytes, p);
  if (s != SI_OK) return s;
  if (!cache || !reused_host) return SI_ERR_NULL;
  if (!cache->x_key || !cache->y_key) return SI_ERR_NULL;
  if (!si::aligned16(cache->x_key) || !si::aligned16(cache->y_key)) return SI_ERR_ALIGN;
  if (std::isnan(gamma)) return SI_ERR_ARG;
  const size_t xbytes = (size_t)p.B * p.C * p.F * (size_t)p.P * p.esize;
  // out may BE the anchor's output buffer: the result then lives there and nothing is copied back and forth
  const bool in_place = out->ptr == cache->y_key;
  const void* held[] = {cache->x_key, cache->y_key};
  for (const void* q : held)
    if (si::ranges_overlap(q, xbytes, x->ptr, xbytes) ||
        (!(in_place && q == cache->y_key) && si::ranges_overlap(q, xbytes, out->ptr, xbytes)) ||
        si::ranges_overlap(q, xbytes, workspace, p.total_bytes))
      return SI_ERR_ARG;
  if (si::ranges_overlap(cache->x_key, xbytes, cache->y_key, xbytes)) return SI_ERR_ARG;

  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  double cosv = std::nan("");
  bool stats_done = false;
  if (cache->valid) {
    // the statistics pass doubles as the similarity pass: x is read once for both
    s = p.dtype == SI_F32
            ? si::launch_gn_stats<float>(p, static_cast<const float*>(x->ptr), static_cast<const float*>(cache->x_key),
                                         w->gn_eps, ws, st)
            : si::launch_gn_stats<si::bf16>(p, static_cast<const si::bf16*>(x->ptr),
                                            static_cast<const si::bf16*>(cache->x_key), w->gn_eps, ws, st);
    if (s != SI_OK) return s;
    const int blocks = p.B * p.F * p.G;
    double* partial = reinterpret_cast<double*>(ws + p.off_rehash);
    double* res = partial + (size_t)blocks * 3;
    {
      si::StageScope scope("cosine_finish", st);
      si::cosine_finish_kernel<<<1, si::kCosBlock, 0, st>>>(partial, blocks, (double)gamma, res,
                                                            reinterpret_cast<int*>(res + 1));
      if (hipGetLastError() != hipSuccess) return SI_ERR_HIP;
    }
    struct { double c; int32_t d; int32_t pad; } host;
    if (hipMemcpyAsync(&host, res, 16, hipMemcpyDeviceToHost, st) != hipSuccess) return SI_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SI_ERR_HIP;
    cosv = host.c;
    stats_done = true;
    if (host.d) {  // similar enough: hand the cached output back, nothing else runs
      if (!in_place) {
        si::StageScope scope("cache_handback", st);
        if (hipMemcpyAsync(out->ptr, cache->y_key, xbytes, hipMemcpyDeviceToDevice, st) != hipSuccess) return SI_ERR_HIP;
      }
      if (cos_host) *cos_host = cosv;
      *reused_host = 1;
      return SI_OK;
    }
  }
  si::pack_record(workspace, si::pack_fingerprint(p, w));
  s = p.dtype == SI_F32 ? si::run_block<float>(p, x, w, ctx, out, ws, st, stats_done)
                        : si::run_block<si::bf16>(p, x, w, ctx, out, ws, st, stats_done);
  if (s != SI_OK) return s;
  {
    si::StageScope scope("cache_update", st);
    if (hipMemcpyAsync(cache->x_key, x->ptr, xbytes, hipMemcpyDeviceToDevice, st) != hipSuccess) return SI_ERR_HIP;
    if (!in_place && hipMemcpyAsync(cache->y_key, out->ptr, xbytes, hipMemcpyDeviceToDevice, st) != hipSuccess)
      return SI_ERR_HIP;
  }
  cache->valid = 1;
  if (cos_host) *cos_host = cosv;
  *reused_host = 0;
  return SI_OK;
}

static int rehash_blocks(int64_t n) {
  // one 16-byte vector per thread per trip, at least 4 trips per thread before adding blocks
  const int64_t vecs = n / 4 + 1;
  int64_t blocks = (vecs + (int64_t)si::kCosBlock * 4 - 1) / ((int64_t)si::kCosBlock * 4);
  if (blocks < 1) blocks = 1;
  if (blocks > si::kCosMaxBlocks) blocks = si::kCosMaxBlocks;
  return (int)blocks;
}

size_t si_rehash_scratch_bytes(int64_t n) {
  if (n < 0) return 0;
  return (size_t)rehash_blocks(n) * 3 * sizeof(double);
}

si_status si_rehash_check(const void* feat_t, const void* feat_prev, int64_t n, int32_t dtype, float thresh,
                          double* cos_dev, int32_t* decision_dev, void* scratch, void* stream) {
  if (n < 0) return SI_ERR_SHAPE;
  if (dtype != SI_F32 && dtype != SI_BF16) return SI_ERR_DTYPE;
  if (std::isnan(thresh)) return SI_ERR_ARG;
  if (!decision_dev || !scratch) return SI_ERR_NULL;
  if (n > 0 && (!feat_t || !feat_prev)) return SI_ERR_NULL;
  if (!si::aligned16(feat_t) || !si::aligned16(feat_prev) || !si::aligned16(scratch)) return SI_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(cos_dev) & 7u) || (reinterpret_cast<uintptr_t>(decision_dev) & 3u)) return SI_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int blocks = rehash_blocks(n);
  double* partial = static_cast<double*>(scratch);
  {
    si::StageScope scope("cosine_partial", st);
    if (dtype == SI_F32)
      si::cosine_partial_kernel<float><<<blocks, si::kCosBlock, 0, st>>>(static_cast<const float*>(feat_t),
                                                                         static_cast<const float*>(feat_prev), n, partial);
    else
      si::cosine_partial_kernel<si::bf16><<<blocks, si::kCosBlock, 0, st>>>(static_cast<const si::bf16*>(feat_t),
                                                                            static_cast<const si::bf16*>(feat_prev), n, partial);
    if (hipGetLastError() != hipSuccess) return SI_ERR_HIP;
  }
  {
    si::StageScope scope("cosine_finish", st);
    si::cosine_finish_kernel<<<1, si::kCosBlock, 0, st>>>(partial, blocks, (double)thresh, cos_dev, decision_dev);
    if (hipGetLastError() != hipSuccess) return SI_ERR_HIP;
  }
  return SI_OK;
}

si_status si_rehash_check_sync(const void* feat_t, const void* feat_prev, int64_t n, int32_t dtype, float thresh,
                               void* scratch, void* result_dev, void* stream, double* cos_host, int32_t* decision_host) {
  if (!result_dev || !cos_host || !decision_host) return SI_ERR_NULL;
  if (!si::aligned16(result_dev)) return SI_ERR_ALIGN;
  double* cos_dev = static_cast<double*>(result_dev);
  int32_t* dec_dev = reinterpret_cast<int32_t*>(static_cast<char*>(result_dev) + 8);
  si_status s = si_rehash_check(feat_t, feat_prev, n, dtype, thresh, cos_dev, dec_dev, scratch, stream);
  if (s != SI_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  struct { double c; int32_t d; int32_t pad; } host;
  if (hipMemcpyAsync(&host, result_dev, 16, hipMemcpyDeviceToHost, st) != hipSuccess) return SI_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return SI_ERR_HIP;
  *cos_host = host.c;
  *decision_host = host.d;
  return SI_OK;
}

#include "si_static_scratch.h"

int32_t si_key_step_search(const float* S, int32_t K, float gamma, int32_t* G_out) {
  if (!S || !G_out || K < 1 || std::isnan(gamma) || gamma > 1.0f) return -1;
  // Algorithm 1 as a scan per anchor: a key step stays the anchor for the run of later steps that are
  // still similar to it; the first step that is not becomes the next key step.  Entries and
  // threshold are compared as the float values the caller passed (a NaN entry counts as dissimilar).
  int32_t count = 0;
  for (int32_t anchor = 0;;) {
    G_out[count++] = anchor;
    if (!(S[(int64_t)anchor * K + anchor] >= gamma)) return -1;  // a step must at least be similar to itself
    int32_t next = anchor + 1;
    while (next < K && S[(int64_t)next * K + anchor] >= gamma) ++next;
    if (next >= K) break;
    anchor = next;
  }
  if (G_out[count - 1] != K - 1) G_out[count++] = K - 1;  // the last step always joins
  return count;
}

void si_stage_timing_enable(int32_t on) { si::g_timing = on != 0; }

int32_t si_stage_timing_read(const char** names, double* total_ms, int64_t* launches, int32_t cap) {
  const int ns = (int)si::g_stage_names.size();
  std::vector<double> ms(ns, 0.0);
  std::vector<int64_t> cnt(ns, 0);
  bool bad = false;
  for (auto& e : si::g_events) {
    float t = 0.f;
    if (hipEventSynchronize(e.b) != hipSuccess || hipEventElapsedTime(&t, e.a, e.b) != hipSuccess) bad = true;
    ms[e.stage] += t;
    cnt[e.stage] += 1;
    (void)hipEventDestroy(e.a);
    (void)hipEventDestroy(e.b);
  }
  si::g_events.clear();
  if (bad) return -1;
  for (int i = 0; i < ns && i < cap; ++i) {
    if (names) names[i] = si::g_stage_names[i].c_str();
    if (total_ms) total_ms[i] = ms[i];
    if (launches) launches[i] = cnt[i];
  }
  return ns;
}

}  // extern "C"
