// C ABI of the ERNIE generation hot path (see include/ernie.h): host-side
// argument checks, arena carving and kernel orchestration.  All device work is
// enqueued on the caller's stream; nothing here allocates device memory.

#include "../../include/ernie.h"
#include "../../include/ernie_debug.h"
#include "../../include/ernie_job.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "attention.h"
#include "common.h"
#include "decode_fused.h"
#include "decode_persist.h"
#include "gemm_prefill.h"
#include "gemm_prefill2.h"
#include "gemm_skinny.h"
#include "handover_probe.h"
#include "rowops.h"

using namespace ernie;

namespace {

constexpr size_t kAlign = 256;
constexpr int kStagingSlots = 8;
constexpr int kFusedMaxBatch = 64;     // the fused-prologue decode path keeps the whole batch in LDS
constexpr int kBigMaxSplitK = 8;       // partial buffers of the raw fp32 GEMM outputs
constexpr size_t kMaxLds = 160 * 1024;
constexpr size_t kPersistMaxLds = kMaxLds - 8 * 1024;
constexpr int kPersistTraceGroups = 512;   // workgroups the time-stamp trace of the one-launch decode kernel has room for

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Per-step temporaries of the small-batch decode step for ernie_decode_step_static: the same buffers the arena
// holds for ernie_decode_step, at the largest shape that entry point accepts.
constexpr int kStaticMaxBatch = 64, kStaticMaxWidth = 1024, kStaticMaxFfn = 4096, kStaticMaxStrips = 1024;
struct StaticLayout {
  static constexpr size_t r_qkv = 0;                                                               // [1][64][3 * 1024] fp32
  static constexpr size_t r_out = r_qkv + (size_t)kStaticMaxBatch * 3 * kStaticMaxWidth * 4;       // [8][64][1024] fp32
  static constexpr size_t r_f2 = r_out + (size_t)kBigMaxSplitK * kStaticMaxBatch * kStaticMaxWidth * 4;   // [4][64][1024] fp32
  static constexpr size_t strip_val = r_f2 + (size_t)4 * kStaticMaxBatch * kStaticMaxWidth * 4;    // [64][1024] fp32
  static constexpr size_t strip_idx = strip_val + (size_t)kStaticMaxBatch * kStaticMaxStrips * 4;  // [64][1024] int32
  static constexpr size_t X = strip_idx + (size_t)kStaticMaxBatch * kStaticMaxStrips * 4;          // [64][1024] fp16
  static constexpr size_t X1 = X + (size_t)kStaticMaxBatch * kStaticMaxWidth * 2;
  static constexpr size_t O = X1 + (size_t)kStaticMaxBatch * kStaticMaxWidth * 2;
  static constexpr size_t hlast = O + (size_t)kStaticMaxBatch * kStaticMaxWidth * 2;
  static constexpr size_t G = hlast + (size_t)kStaticMaxBatch * kStaticMaxWidth * 2;               // [64][4096] fp16
  static constexpr size_t total = G + (size_t)kStaticMaxBatch * kStaticMaxFfn * 2;
};
static_assert(StaticLayout::total == 5 * 1024 * 1024 + 256 * 1024, "5.25 MiB of static device memory per GPU");

struct LayerPtrs {
  half_t *wqkv, *wo, *w1, *w2;                       // fragment-major
  float *bqkv, *bo, *b1, *b2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
};

// Offsets of every sub-buffer inside the arena (bytes).  Computed identically
// for sizing (arena == NULL) and for carving.
struct ArenaPlan {
  size_t tok_rm, tok_p, pos, emb_g, emb_b, kept;
  struct L { size_t wqkv, wo, w1, w2, bqkv, bo, b1, b2, ln1_g, ln1_b, ln2_g, ln2_b; };
  std::vector<L> layers;
  size_t r_qkv, r_out, r_f1, r_f2, zero_bias;
  size_t type_emb, head_w, head_b, head_g, head_beta, out_bias;   // optional variants (0 bytes when off)
  bool has_type, has_head, has_bias;
  size_t kv, X, X1, Y, Q, O, G, Yf, hlast, strip_val, strip_idx, cu, lens, tok_seq, tok_pos, tok_prev;
  size_t finished, slot, keep, r_logits;
  size_t xch, ptab, epoch, trace;        // one-launch decode step: exchange buffers, layer table, step counter
  PersistXch xo; int xch_batch;          // offsets inside a layer's exchange region and its row capacity (0 = none)
  size_t total;
  int vocab_tiles, strips;
  size_t t_max;
};

ArenaPlan make_plan(const ErnieConfig& c, const ErnieVariants* var) {
  ArenaPlan p;
  p.has_type = var && var->type_emb;
  p.has_head = var && var->head_w;
  p.has_bias = var && var->out_bias;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t d = c.d_model, f = c.d_ffn, V = c.vocab_kept, P = c.max_pos;
  p.vocab_tiles = (int)((V + 31) / 32);
  p.strips = p.vocab_tiles;
  p.tok_rm = take(V * d * 2);
  p.tok_p = take((size_t)p.vocab_tiles * 32 * d * 2);
  p.pos = take(P * d * 2);
  p.emb_g = take(d * 4);
  p.emb_b = take(d * 4);
  p.kept = take(V * 4);
  p.layers.resize(c.n_layers);
  for (auto& l : p.layers) {
    l.wqkv = take(3 * d * d * 2); l.wo = take(d * d * 2); l.w1 = take(f * d * 2); l.w2 = take(d * f * 2);
    l.bqkv = take(3 * d * 4); l.bo = take(d * 4); l.b1 = take(f * 4); l.b2 = take(d * 4);
    l.ln1_g = take(d * 4); l.ln1_b = take(d * 4); l.ln2_g = take(d * 4); l.ln2_b = take(d * 4);
  }
  const size_t Bm = c.max_batch, S = c.max_seq;
  p.kv = take((size_t)c.n_layers * 2 * Bm * S * d * 2);
  const size_t lmax = (size_t)(c.max_seq < c.max_pos ? c.max_seq : c.max_pos);
  p.t_max = Bm * lmax;
  p.X = take(p.t_max * d * 2); p.X1 = take(p.t_max * d * 2); p.Y = take(p.t_max * d * 2);
  p.Q = take(p.t_max * d * 2); p.O = take(p.t_max * d * 2); p.G = take(p.t_max * f * 2);
  p.Yf = take(Bm * d * 4);
  // raw fp32 GEMM outputs of the decode step, split over K into up to kBigMaxSplitK partial buffers
  p.r_qkv = take((size_t)kBigMaxSplitK * Bm * 3 * d * 4); p.r_out = take((size_t)kBigMaxSplitK * Bm * d * 4);
  p.r_f1 = take((size_t)kBigMaxSplitK * Bm * f * 4); p.r_f2 = take((size_t)kBigMaxSplitK * Bm * d * 4);
  p.zero_bias = take(std::max(std::max(3 * d, f), V) * 4);
  // fp32 partial logits of the large-batch projection (two splits at most); not needed while max_batch <= 64
  p.r_logits = take(Bm > 64 ? (size_t)2 * Bm * V * 4 : 0);
  p.type_emb = take(p.has_type ? 2 * d * 2 : 0);
  p.head_w = take(p.has_head ? d * d * 2 : 0);
  p.head_b = take(p.has_head ? d * 4 : 0); p.head_g = take(p.has_head ? d * 4 : 0);
  p.head_beta = take(p.has_head ? d * 4 : 0);
  p.out_bias = take(p.has_bias ? V * 4 : 0);
  p.hlast = take(Bm * d * 2);
  p.strip_val = take(Bm * p.strips * 4); p.strip_idx = take(Bm * p.strips * 4);
  p.cu = take((Bm + 1) * 4); p.lens = take(Bm * 4);
  p.tok_seq = take(p.t_max * 4); p.tok_pos = take(p.t_max * 4); p.tok_prev = take(Bm * 4);
  p.finished = take(Bm * 4); p.slot = take(Bm * 4); p.keep = take(Bm * 4);
  // exchange buffers of the one-launch decode step (pairs of fp16 + tag: 4 bytes per element), one set per layer
  p.xch_batch = (d <= 1024 && f <= 4096) ? (int)std::min<size_t>(Bm, kFusedMaxBatch) : 0;
  {
    const size_t xb = (size_t)p.xch_batch * 4;
    p.xo.qkv = 0; p.xo.o = (unsigned)(xb * 3 * d); p.xo.y1 = p.xo.o + (unsigned)(xb * d);
    p.xo.g = p.xo.y1 + (unsigned)(xb * d); p.xo.y2 = p.xo.g + (unsigned)(xb * f); p.xo.x = p.xo.y2 + (unsigned)(xb * d);
    p.xo.x1 = p.xo.x + (unsigned)(xb * d); p.xo.layer_bytes = (unsigned)align_up(p.xo.x1 + xb * d);
    p.xch = take((size_t)p.xo.layer_bytes * c.n_layers);
    p.ptab = take(p.xch_batch ? sizeof(PersistLayer) * c.n_layers : 0);
    p.epoch = take(256);
    p.trace = take(p.xch_batch ? (size_t)kPersistTraceGroups * c.n_layers * 32 * 8 : 0);
  }
  p.total = off;
  return p;
}

int check_config(const ErnieConfig* c) {
  if (!c) return ERNIE_EINVAL;
  if (c->n_layers < 1 || c->d_model < 64 || c->n_heads < 1 || c->d_ffn < 64) return ERNIE_EINVAL;
  if (c->d_model != c->n_heads * kHeadDim) return ERNIE_EINVAL;          // head_dim must be 64
  if (c->d_model > 64 * 8 * kMaxRowChunks) return ERNIE_EINVAL;           // one wave normalises a row
  if (c->d_ffn % 64 != 0) return ERNIE_EINVAL;
  if (c->vocab_kept < 1 || c->vocab_full < c->vocab_kept || c->max_pos < 1) return ERNIE_EINVAL;
  if (c->max_batch < 1 || c->max_batch > 256 || c->max_seq < 1) return ERNIE_EINVAL;
  if (!(c->ln_eps > 0.f)) return ERNIE_EINVAL;
  return ERNIE_OK;
}

}  // namespace

// File-scope device array behind ernie_decode_step_static.  In host code this name is only a stand-in for the
// symbol: the device address is looked up once per device (static_scratch_for_current_device) and that
// pointer is what kernels and copies receive.
static __device__ __align__(256) unsigned char scratch[StaticLayout::total];

// Optional per-kernel timing (ernie_profile): HIP events recorded on the caller's stream
// around every launch of a category, plus the algorithmic bytes / flops of those launches.
struct ProfSlot { hipEvent_t a, b; int cat; };
struct Profiler {
  bool on = false;
  std::vector<ProfSlot> slots;
  size_t used = 0;
  double bytes[ERNIE_PROF_NCAT] = {0}, flops[ERNIE_PROF_NCAT] = {0};
};

struct ErnieHandle {
  ErnieConfig cfg;
  Profiler prof;
  double sum_len, sum_len2;   // over the batch in flight: sum of prompt lengths and of their squares
  ArenaPlan plan;
  unsigned char* arena;
  half_t *tok_rm, *tok_p, *pos;
  float *emb_g, *emb_b;
  std::vector<LayerPtrs> layers;
  half_t *kv, *X, *X1, *Y, *Q, *O, *G, *hlast;
  float *Yf, *strip_val, *r_qkv, *r_out, *r_f1, *r_f2, *zero_bias;
  half_t *type_emb = nullptr, *head_w = nullptr;                      // optional variants, null when off
  float *head_b = nullptr, *head_g = nullptr, *head_beta = nullptr, *out_bias = nullptr;
  int sk_out, sk_f2, fused_decode, attn_dec, attn_nt = 1, ln_ns = 0, ln_rpw = 0, big_f1_fused = 1, big_logits_gemm = 1, dec_nw16 = 2, dec_prefetch = 64, kv_prefetch = 1, big_warm = 16, pf_tile = 0, big_ln_rows = 1, big_f1_tile = 0, big_narrow = 1, big_mfast = 1;
  int cand = 0;                  // argmax candidates per row left by the last projection   // decode tuning (see ernie_debug_tune)
  int *strip_idx, *cu, *lens, *tok_seq, *tok_pos, *tok_prev;
  float* r_logits = nullptr;     // [2][max_batch][V'] fp32, large-batch projection only
  int *finished, *slot, *keep;   // per-sequence finished flag, cache row of each batch row, compaction list
  int eos = -1;                  // end-of-sequence id (trimmed), -1 = none
  bool compacted = false;        // some row map entry differs from its index
  std::vector<int> row_len;      // host copy of the prompt lengths of the batch in flight
  // Pinned host staging for the small host arrays of prefill / compact: kStagingSlots slots used round-robin by
  // eager calls (a slot is reused only after the copy that read it has executed: one event per slot), then
  // kStagingSlots slots handed out once each to calls made under stream capture (a replayed graph reads its
  // slot again, so it is never reused).  Each slot holds max_batch + 1 ints.
  int* staging;
  int staging_next, staging_captured;
  hipEvent_t stage_ev[kStagingSlots];
  bool stage_busy[kStagingSlots];
  // state of the batch in flight
  bool prefilled;
  int B, max_len, steps;
  unsigned char* static_scratch = nullptr;
  // one-launch decode step (decode_persist.h)
  int persist = 1, persist_stall = 0, persist_trace = 0, persist_dbg = 0, persist_helpers = 1, cu_count = 0;
  unsigned persist_spin = 1u << 17;
  unsigned char* xch = nullptr; PersistLayer* ptab = nullptr; unsigned* epoch = nullptr;
  std::vector<PersistLayer> ptab_host;   // source of the asynchronous copy into `ptab`: lives as long as the handle
  int* err_host = nullptr;               // pinned, device-visible: a bounded wait that gave up leaves 1 here   // device address of the file-scope scratch array on this handle's GPU
};

// Device address of the file-scope `scratch` array on the CURRENT device, looked up once per device and kept:
// every GPU holds its own copy of the array at its own address.
static int static_scratch_for_current_device(unsigned char** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static unsigned char* ptr_of_device[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ERNIE_EHIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return ERNIE_EHIP; }
    ptr_of_device[dev] = static_cast<unsigned char*>(p);
  }
  *out = ptr_of_device[dev];
  return ERNIE_OK;
}

// A staging slot for one host -> device copy on stream `s`; *slot_out is the ring slot to pass to
// stage_release after the copy has been enqueued, or -1 for a capture slot.  Returns null when the stream is
// capturing and the capture slots are used up.
static int* stage_acquire(ErnieHandle* h, hipStream_t s, int* slot_out) {
  const size_t pitch = (size_t)h->cfg.max_batch + 1;
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); st = hipStreamCaptureStatusNone; }
  if (st == hipStreamCaptureStatusActive) {
    *slot_out = -1;
    if (h->staging_captured >= kStagingSlots) return nullptr;
    return h->staging + (size_t)(kStagingSlots + h->staging_captured++) * pitch;
  }
  const int slot = h->staging_next;
  h->staging_next = (slot + 1) % kStagingSlots;
  if (h->stage_busy[slot]) { (void)hipEventSynchronize(h->stage_ev[slot]); h->stage_busy[slot] = false; }
  *slot_out = slot;
  return h->staging + (size_t)slot * pitch;
}

static void stage_release(ErnieHandle* h, hipStream_t s, int slot) {
  if (slot < 0) return;
  if (hipEventRecord(h->stage_ev[slot], s) == hipSuccess) h->stage_busy[slot] = true;
  else { (void)hipGetLastError(); (void)hipStreamSynchronize(s); }      // no event: wait for the copy instead
}

namespace {

// Row-kernel instantiation by model width: RC chunks of 512 features per wave.
#define ROW_DISPATCH(d, CALL) do { if ((d) <= 1024) { constexpr int RC = 2; CALL; } else if ((d) <= 2048) { constexpr int RC = 4; CALL; } else { constexpr int RC = 8; CALL; } } while (0)

// Brackets one launch with events when profiling is on (no-op otherwise).
struct ProfScope {
  ErnieHandle* h; hipStream_t s; long idx;
  ProfScope(ErnieHandle* h_, int cat, hipStream_t s_, double bytes, double flops) : h(h_), s(s_), idx(-1) {
    Profiler& p = h->prof;
    if (!p.on || p.used >= p.slots.size()) return;
    idx = (long)p.used++;
    p.slots[idx].cat = cat;
    p.bytes[cat] += bytes; p.flops[cat] += flops;
    (void)hipEventRecord(p.slots[idx].a, s);
  }
  ~ProfScope() { if (idx >= 0) (void)hipEventRecord(h->prof.slots[idx].b, s); }
};

#define HIP_OK(expr) do { if ((expr) != hipSuccess) return ERNIE_EHIP; } while (0)

int launch_status() { return hipGetLastError() == hipSuccess ? ERNIE_OK : ERNIE_EHIP; }

half_t* kcache(const ErnieHandle* h, int layer) {
  const size_t per = (size_t)h->cfg.max_batch * h->cfg.max_seq * h->cfg.d_model;
  return h->kv + ((size_t)layer * 2 + 0) * per;
}
half_t* vcache(const ErnieHandle* h, int layer) {
  const size_t per = (size_t)h->cfg.max_batch * h->cfg.max_seq * h->cfg.d_model;
  return h->kv + ((size_t)layer * 2 + 1) * per;
}

// Decode attention: (waves, groups in flight per wave) chosen so that one batch of NW * U * 8 keys covers
// the whole cache when the capacity allows it (a single memory round trip); long caches stream with 4 waves.
void launch_attn_decode(const ErnieHandle* h, const float* rqkv, int sk_in, int B, const float* bqkv, half_t* kc,
                        half_t* vc, hipStream_t s, DecPrefetch warm = DecPrefetch{}) {
  const int H = h->cfg.n_heads, S = h->cfg.max_seq, d = h->cfg.d_model;
  // warming workgroups: whole extra grid rows, a multiple of 8 workgroups (consecutive ids, one per XCD)
  int extra_rows = 0;
  if (warm.count > 0 && (warm.aux[0] || warm.aux[1])) {
    extra_rows = (warm.count + H - 1) / H;
    while ((extra_rows * H) % 8 != 0) ++extra_rows;
  }
  warm.count = extra_rows * H;
  int v = h->attn_dec;
  // Measured on all benchmark shapes: two key groups in flight per wave (84 registers, five waves per SIMD)
  // beat four (115 registers) by 0.3-3 %; with thousands of short streams (B x H >= 1024, capacity <= 384
  // positions) two waves per workgroup beat four by another 1.7 %.
  if (v == 0) v = ((long)B * H >= 1024 && S <= 384) ? 5 : 4;
#define ATTN_DEC_LAUNCH(NW, U, NT)                                                                                  \
  hipLaunchKernelGGL((attn_decode_fused_kernel<NW, U, NT>), dim3(H, B + extra_rows), dim3(NW * 64), 0, s, rqkv, sk_in, B, bqkv, \
                     kc, vc, h->lens, H, S, d, h->O, h->eos >= 0 ? h->finished : nullptr,                        \
                     h->compacted ? h->slot : nullptr, warm)
  if (v == 2) ATTN_DEC_LAUNCH(8, 3, false);
  else if (v == 3) ATTN_DEC_LAUNCH(8, 4, false);
  else if (v == 4) ATTN_DEC_LAUNCH(4, 2, true);
  else if (v == 5) ATTN_DEC_LAUNCH(2, 2, true);
  else if (h->attn_nt) ATTN_DEC_LAUNCH(4, 4, true);
  else ATTN_DEC_LAUNCH(4, 4, false);
#undef ATTN_DEC_LAUNCH
}

// Tile shape by problem size: large tiles halve the L2 -> LDS bytes per flop but need enough of them
// to fill 256 CUs twice over; small problems take smaller tiles so that every CU holds several workgroups.
template <int WGM, int WGN, int TM, int TN, int BK, int S, class Epi>
void launch_gemm_prefill_t(const half_t* A, const half_t* Wp, const float* bias, int M, int N, int K, Epi epi,
                           hipStream_t s, bool rows_fastest = false) {
  using P = GemmPipe<WGM, WGN, TM, TN, BK, S>;
  const int tiles_m = (M + P::kBM - 1) / P::kBM, tiles_n = (N + P::kBN - 1) / P::kBN;
  hipLaunchKernelGGL((gemm_prefill2_kernel<WGM, WGN, TM, TN, BK, S, Epi>), dim3(tiles_m * tiles_n), dim3(64 * WGM * WGN),
                     P::kLdsBytes, s,
                     A, Wp, bias, M, N, K, (N + 31) / 32, rows_fastest ? -tiles_m : tiles_n, epi);
}

template <class Epi>
void launch_gemm_prefill(ErnieHandle* h, const half_t* A, const half_t* Wp, const float* bias, int M, int N, int K,
                         Epi epi, hipStream_t s, int category = ERNIE_PROF_GEMM_PREFILL) {
  ProfScope prof(h, category, s, 2.0 * N * K, 2.0 * M * N * K);
  const long tiles_256x256 = (long)((M + 255) / 256) * ((N + 255) / 256);
  const long tiles_128x128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  // 256 x 256 when there are at least two rounds of them over the 256 CUs, or a single round that fills at
  // least half the CUs (one tile per CU beats several rounds of smaller tiles); 128 x 128 when they fill the
  // chip one and a half times; otherwise 64 x 64 with BK = 64 (measured 3-15 % faster than 128 x 64 there).
  const int forced = h->pf_tile;          // test hook: 1 / 2 / 3 force the 256 / 128 / 64 tile
  if (forced == 1 || (!forced && (tiles_256x256 >= 512 || (tiles_256x256 >= 128 && tiles_256x256 <= 256))))
    launch_gemm_prefill_t<4, 4, 2, 2, 64, 2>(A, Wp, bias, M, N, K, epi, s);
  else if (forced == 2 || (!forced && tiles_128x128 >= 384)) launch_gemm_prefill_t<2, 2, 2, 2, 32, 3>(A, Wp, bias, M, N, K, epi, s);
  else launch_gemm_prefill_t<2, 2, 1, 1, 64, 3>(A, Wp, bias, M, N, K, epi, s);
}

template <int MT, int NW>
void launch_logits_t(ErnieHandle* h, const half_t* X, int B, float* logits_out, hipStream_t s) {
  const size_t lds = (size_t)NW * MT * 16 * 64 * 4;
  hipLaunchKernelGGL((logits_argmax_kernel<MT, NW>), dim3(h->plan.strips), dim3(NW * 64), lds, s, X, h->tok_p, B,
                     h->cfg.vocab_kept, h->cfg.d_model, h->out_bias, logits_out, h->strip_val, h->strip_idx,
                     h->plan.strips);
}

void launch_logits_big(ErnieHandle* h, const half_t* X, int B, float* logits_out, hipStream_t s);

// Leaves per-strip argmax candidates in strip_val / strip_idx; returns how many candidates each row has.
int launch_logits(ErnieHandle* h, const half_t* X, int B, float* logits_out, hipStream_t s) {
  // (the GEMM epilogue stores runs of 8 columns, so the row length must be a multiple of 8; the row kernel
  // writes the caller's logits in 16-byte pieces)
  if (B > 64 && h->big_logits_gemm && h->cfg.vocab_kept % 8 == 0 && (uintptr_t)logits_out % 16 == 0) {
    launch_logits_big(h, X, B, logits_out, s);
    return 1;
  }
  if (B <= 32) launch_logits_t<1, 4>(h, X, B, logits_out, s);
  else if (B <= 64) launch_logits_t<2, 4>(h, X, B, logits_out, s);
  else if (B <= 128) launch_logits_t<4, 4>(h, X, B, logits_out, s);
  else launch_logits_t<8, 4>(h, X, B, logits_out, s);
  return h->plan.strips;
}

// Kernels whose dynamic LDS exceeds the 64 KiB default need an explicit opt-in.
template <class F>
int allow_lds(F* fn, size_t bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes) == hipSuccess ? ERNIE_OK : ERNIE_EHIP;
}

int configure_kernels() {
  int rc = ERNIE_OK;
#define GEMM_LDS(...)                                                                              \
  rc |= allow_lds(gemm_prefill2_kernel<__VA_ARGS__, EpiQKV>, GemmPipe<__VA_ARGS__>::kLdsBytes);       \
  rc |= allow_lds(gemm_prefill2_kernel<__VA_ARGS__, EpiResidual>, GemmPipe<__VA_ARGS__>::kLdsBytes);  \
  rc |= allow_lds(gemm_prefill2_kernel<__VA_ARGS__, EpiGelu>, GemmPipe<__VA_ARGS__>::kLdsBytes);      \
  rc |= allow_lds(gemm_prefill2_kernel<__VA_ARGS__, EpiRaw32>, GemmPipe<__VA_ARGS__>::kLdsBytes)
  GEMM_LDS(4, 4, 2, 2, 64, 2); GEMM_LDS(2, 2, 2, 2, 32, 3); GEMM_LDS(2, 2, 1, 1, 64, 3);
#undef GEMM_LDS
  rc |= allow_lds(gemm_prefill2_kernel<2, 2, 1, 1, 64, 3, EpiGeluFast>, GemmPipe<2, 2, 1, 1, 64, 3>::kLdsBytes);
  const size_t big = (size_t)4 * 8 * 16 * 64 * 4;   // MT = 8, NW = 4
  rc |= allow_lds(logits_argmax_kernel<8, 4>, big);
#define LN_LDS2(NW, EPI, SK, RPW) rc |= allow_lds(gemm_dec_ln_kernel<NW, EPI, 2, SK, RPW, 1>, kMaxLds); rc |= allow_lds(gemm_dec_ln_kernel<NW, EPI, 2, SK, RPW, 2>, kMaxLds); rc |= allow_lds(gemm_dec_ln_kernel<NW, EPI, 2, SK, RPW, 4>, kMaxLds)
#define LN_LDS1(EPI, SK, RPW) LN_LDS2(8, EPI, SK, RPW)
#define LN_LDS(EPI, SK) LN_LDS1(EPI, SK, 1); LN_LDS1(EPI, SK, 2)
  LN_LDS(EPI_RAW, 0);
  LN_LDS(EPI_RAW, 1); LN_LDS(EPI_RAW, 2); LN_LDS(EPI_RAW, 4); LN_LDS(EPI_GELU16, 1); LN_LDS(EPI_GELU16, 2); LN_LDS(EPI_GELU16, 4);
#undef LN_LDS
#undef LN_LDS1
#undef LN_LDS2
  // (the one-launch kernel also holds a few KB of statically declared LDS)
#define PERSIST_LDS(RPW) rc |= allow_lds(decode_persist_kernel<RPW, 6, 24, 6>, kPersistMaxLds); rc |= allow_lds(decode_persist_kernel<RPW, 8, 8, 6>, kPersistMaxLds); \
  rc |= allow_lds(decode_persist_kernel<RPW, 8, 16, 6>, kPersistMaxLds); rc |= allow_lds(decode_persist_kernel<RPW, 8, 24, 6>, kPersistMaxLds); \
  rc |= allow_lds(decode_persist_kernel<RPW, 8, 32, 6>, kPersistMaxLds)
  PERSIST_LDS(1); PERSIST_LDS(2);
#undef PERSIST_LDS
  rc |= allow_lds(gemm_dec_kernel<1, 8, EPI_RAW>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<1, 16, EPI_RAW>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<1, 16, EPI_ARGMAX>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<2, 16, EPI_RAW>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<2, 16, EPI_ARGMAX>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<2, 8, EPI_RAW>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<1, 8, EPI_ARGMAX>, kMaxLds);
  rc |= allow_lds(gemm_dec_kernel<2, 8, EPI_ARGMAX>, kMaxLds);
  return rc ? ERNIE_EHIP : ERNIE_OK;
}


// Split of the contraction over `gridDim.y` workgroups for the GEMMs with few
// column strips: the smallest divisor of the k-tile count that brings the grid
// to about 96 workgroups, capped so that the consumer does not pay for many partials.
int pick_split_k(int strips, int k_tiles, int cap) {
  int best = 1;
  for (int sk = 1; sk <= cap; sk *= 2) {          // 1, 2, 4: the splits the consumers are instantiated for
    if (k_tiles % sk != 0 || k_tiles / sk < 8) continue;
    best = sk;
    if (strips * sk >= 96) break;
  }
  return best;
}

size_t dec_lds_bytes(int MT, int NW, int kslice) {
  const size_t a = (size_t)MT * 32 * (kslice + 8) * 2, r = (size_t)NW * MT * 16 * 64 * 4;
  return a > r ? a : r;
}

template <int EPI>
int launch_gemm_dec(ErnieHandle* h, DecGemmArgs a, int sk, hipStream_t s) {
  ProfScope prof(h, EPI == EPI_ARGMAX ? ERNIE_PROF_LOGITS : ERNIE_PROF_GEMM_DEC, s, 2.0 * a.N * a.K, 2.0 * a.B * a.N * a.K);
  const int MT = (a.B + 31) / 32;
  if (sk < 1 || (a.K / 16) % sk != 0) return ERNIE_EINVAL;
  const int kslice = a.K / sk;
  a.n_main = (a.N + 31) / 32;
  // warming workgroups: extra columns of the grid, a multiple of 8 per split (ranks 8 j .. 8 j + 7 then have
  // consecutive linear ids, i.e. one per XCD)
  int extra = 0;
  const int want_pf = a.pf.ptr ? (a.pf.count + 7) / 8 * 8 : 0, want_kv = a.kv.k ? a.kv.count : 0;
  if (want_pf + want_kv > 0) extra = ((want_pf + want_kv + sk - 1) / sk + 7) / 8 * 8;
  a.pf.count = want_kv ? want_pf : extra * sk;
  a.kv.count = want_kv ? extra * sk - want_pf : 0;
  if (!a.pf.count) a.pf.ptr = nullptr;
  if (!a.kv.count) a.kv.k = nullptr;
  const dim3 grid(a.n_main + extra, sk);
#define DEC_LAUNCH(MTV, NWV)                                                                    \
  do {                                                                                          \
    const size_t lds = dec_lds_bytes(MTV, NWV, kslice);                                         \
    if (lds > kMaxLds) return ERNIE_EINVAL;                                                     \
    hipLaunchKernelGGL((gemm_dec_kernel<MTV, NWV, EPI>), grid, dim3(NWV * 64), lds, s, a);      \
  } while (0)
  const int tiles_wg = a.K / 16 / sk;
  const bool nw16 = tiles_wg >= 16 &&
                    (h->dec_nw16 >= 3 || (h->dec_nw16 == 2 && EPI == EPI_RAW) || (h->dec_nw16 == 1 && EPI == EPI_RAW && a.K >= 2048));
  if (nw16 && MT == 1) DEC_LAUNCH(1, 16);
  else if (nw16 && MT == 2) DEC_LAUNCH(2, 16);
  else if (MT == 1) DEC_LAUNCH(1, 8);
  else if (MT == 2) DEC_LAUNCH(2, 8);
  else return ERNIE_EINVAL;
#undef DEC_LAUNCH
  return ERNIE_OK;
}

template <int EPI, int NW>
int launch_gemm_dec_ln_nw(ErnieHandle* h, DecGemmArgs a, int ns, int rpw, hipStream_t s) {
  const int R = NW * rpw;
  const size_t a_bytes = (size_t)R * (a.K + 8) * 2, r_bytes = (size_t)NW * ns * (R / 2) * 64 * 4;
  const size_t lds = a_bytes > r_bytes ? a_bytes : r_bytes;
  if (lds > kMaxLds) return ERNIE_EINVAL;
  const int strips = (a.N + 31) / 32;
  a.n_main = ((strips + ns - 1) / ns) * ((a.B + R - 1) / R);
  if (!a.kv.k || a.kv.count <= 0) { a.kv.k = nullptr; a.kv.count = 0; }
  a.kv.count = (a.kv.count + 7) / 8 * 8;
  const dim3 grid(a.n_main + a.kv.count), block(NW * 64);
#define LN_LAUNCH(SK, RPW, NS) hipLaunchKernelGGL((gemm_dec_ln_kernel<NW, EPI, 2, SK, RPW, NS>), grid, block, lds, s, a)
#define LN_BY_NS(SK, RPW) do { if (ns == 1) LN_LAUNCH(SK, RPW, 1); else if (ns == 2) LN_LAUNCH(SK, RPW, 2); else LN_LAUNCH(SK, RPW, 4); } while (0)
#define LN_BY_RPW(SK) do { if (rpw == 1) LN_BY_NS(SK, 1); else LN_BY_NS(SK, 2); } while (0)
  switch (a.sk_in) {      // the count of split-K partials to add is a template parameter of the prologue
    case 0: if constexpr (EPI == EPI_RAW) { LN_BY_RPW(0); break; } else return ERNIE_EINVAL;   // embedding prologue
    case 1: LN_BY_RPW(1); break;
    case 2: LN_BY_RPW(2); break;
    case 4: LN_BY_RPW(4); break;
    default: return ERNIE_EINVAL;
  }
#undef LN_BY_RPW
#undef LN_BY_NS
#undef LN_LAUNCH
  return ERNIE_OK;
}

// Two strips per workgroup halve the redundant prologue traffic; the batch is cut into four row groups
// (8 rows per group up to B = 32, one row per wave; 16 rows per group above, two rows per wave).  Measured:
// 8 % over one strip at B = 32, 6 % over one strip x 8-row groups at B = 64; every other combination of
// 1/2/4 strips and 8/16/32 rows is slower at both sizes.  The knobs override the choice (0 = automatic).
void ln_gemm_shape(const ErnieHandle* h, int B, int* ns, int* rpw) {
  *ns = h->ln_ns ? h->ln_ns : 2;
  *rpw = h->ln_rpw ? h->ln_rpw : (B > 32 ? 2 : 1);
}

template <int EPI>
int launch_gemm_dec_ln(ErnieHandle* h, DecGemmArgs a, hipStream_t s) {
  ProfScope prof(h, ERNIE_PROF_GEMM_DEC_LN, s, 2.0 * a.N * a.K, 2.0 * a.B * a.N * a.K);
  if (a.K > 1024) return ERNIE_EINVAL;                 // the LayerNorm prologue holds rows of <= 1024 features
  int ns, rpw;
  ln_gemm_shape(h, a.B, &ns, &rpw);
  return launch_gemm_dec_ln_nw<EPI, 8>(h, a, ns, rpw, s);   // sixteen waves measured 6-30 % slower here
}

// Registers the float vectors first .. last_end (one run of the arena: the per-layer vectors are carved
// back to back) as small-vector region `slot` of a warm-up; a run that is not the expected few KB (at most
// 1 MiB, a multiple of 16 bytes) is skipped.
void set_aux(DecPrefetch& f, int slot, const float* first, const float* last_end) {
  const ptrdiff_t bytes = reinterpret_cast<const unsigned char*>(last_end) - reinterpret_cast<const unsigned char*>(first);
  if (bytes <= 0 || bytes > (ptrdiff_t)1 << 20 || bytes % 16 != 0) return;
  f.aux[slot] = reinterpret_cast<const unsigned char*>(first);
  f.aux_bytes[slot] = (unsigned)bytes;
}

// Warm-up descriptor (see DecPrefetch) for the weights [N, K] of the LayerNorm-prologue GEMM that runs next.
DecPrefetch prefetch_for(const ErnieHandle* h, const half_t* Wp, int N, int K, int B) {
  DecPrefetch f{};
  if (h->dec_prefetch <= 0 || (N % 32) != 0) return f;
  int ns, rpw;
  ln_gemm_shape(h, B, &ns, &rpw);
  const int R = 8 * rpw;
  f.ptr = reinterpret_cast<const unsigned char*>(Wp);
  f.strip_bytes = (unsigned)K * 64u; f.n_strips = N / 32; f.count = h->dec_prefetch;
  f.cons_ns = ns; f.cons_zg = (B + R - 1) / R; f.cons_grid = ((f.n_strips + ns - 1) / ns) * f.cons_zg;
  return f;
}

// Warm-up descriptor (see KvPrefetch) for the cache rows that layer `l`'s decode attention of this step will stream.
KvPrefetch kv_prefetch_for(const ErnieHandle* h, int l, int B) {
  KvPrefetch f{};
  const int H = h->cfg.n_heads;
  if (!h->kv_prefetch) return f;
  f.k = reinterpret_cast<const unsigned char*>(kcache(h, l)); f.v = reinterpret_cast<const unsigned char*>(vcache(h, l));
  f.slot = h->compacted ? h->slot : nullptr;
  f.B = B; f.H = H; f.S = h->cfg.max_seq;
  f.rows = std::min(h->cfg.max_seq, h->max_len + h->steps);
  // two (sequence, head) streams per warming workgroup measured best at B = 32 (more contend with the host
  // kernel, fewer outlast it)
  f.count = h->kv_prefetch > 1 ? h->kv_prefetch : (H * B / 2 + 7) / 8 * 8;
  return f;
}

// Small batches: every GEMM input fits in LDS, row-wise work lives in consumer prologues (5 launches per layer).
bool fused_decode_fits(const ErnieHandle* h, int B) {
  if (!h->fused_decode || B > kFusedMaxBatch || h->cfg.d_model > 1024) return false;
  const int MT = (B + 31) / 32, d = h->cfg.d_model, f = h->cfg.d_ffn;
  return dec_lds_bytes(MT, 8, d) <= kMaxLds && dec_lds_bytes(MT, 8, f / h->sk_f2) <= kMaxLds &&
         (d / 16) % h->sk_out == 0 && (f / 16) % h->sk_f2 == 0;
}

const half_t* apply_head(ErnieHandle* h, const half_t* x, int B, hipStream_t s);

int decode_layers_fused(ErnieHandle* h, const int* tok, float* logits_out, float* hidden_out, hipStream_t s) {
  const ErnieConfig& c = h->cfg;
  const int B = h->B, d = c.d_model, f = c.d_ffn;
  int rc = ERNIE_OK;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerPtrs& L = h->layers[l];
    DecGemmArgs a{};
    a.B = B; a.eps = c.ln_eps;
    // QKV: layer 0 reads the embedding rows; later layers normalise the previous FFN2 output on the fly
    a.Wp = L.wqkv; a.N = 3 * d; a.K = d; a.rout = h->r_qkv;
    if (l == 0) {
      // the embedding LayerNorm of the fed tokens is this GEMM's prologue (no separate embedding launch)
      a.sk_in = 0; a.tok = tok; a.cache_len = h->lens; a.tok_emb = h->tok_rm; a.pos_emb = h->pos;
      a.seg_row = h->type_emb ? h->type_emb + d : nullptr; a.max_pos = c.max_pos; a.vocab_kept = c.vocab_kept; a.eos = h->eos; a.finished = h->finished;
      a.gamma = h->emb_g; a.beta = h->emb_b; a.xout = h->X;
      a.kv = kv_prefetch_for(h, l, B);
      rc |= launch_gemm_dec_ln<EPI_RAW>(h, a, s);
    } else {
      const LayerPtrs& P = h->layers[l - 1];
      a.r32 = h->r_f2; a.sk_in = h->sk_f2; a.bias = P.b2; a.res = h->X1; a.gamma = P.ln2_g; a.beta = P.ln2_b;
      a.xout = h->X;
      a.kv = kv_prefetch_for(h, l, B);
      rc |= launch_gemm_dec_ln<EPI_RAW>(h, a, s);
    }
    {
      // K and V of every visible position (cached + the appended one), 2 bytes each
      ProfScope prof(h, ERNIE_PROF_ATTN_DEC, s, 2.0 * (h->sum_len + (double)B * (h->steps + 1)) * d * 2.0, 0.0);
      launch_attn_decode(h, h->r_qkv, 1, B, L.bqkv, kcache(h, l), vcache(h, l), s);
    }
    DecGemmArgs o{};
    o.B = B; o.Wp = L.wo; o.N = d; o.K = d; o.a16 = h->O; o.rout = h->r_out;
    // FFN1 comes next: its weights, and bo, b1, b2, ln1 scale / shift (contiguous in the arena)
    o.pf = prefetch_for(h, L.w1, f, d, B);
    if (o.pf.ptr) set_aux(o.pf, 0, L.bo, L.ln1_b + d);
    rc |= launch_gemm_dec<EPI_RAW>(h, o, h->sk_out, s);
    DecGemmArgs f1{};
    f1.B = B; f1.eps = c.ln_eps; f1.Wp = L.w1; f1.N = f; f1.K = d; f1.r32 = h->r_out; f1.sk_in = h->sk_out;
    f1.bias = L.bo; f1.res = h->X; f1.gamma = L.ln1_g; f1.beta = L.ln1_b; f1.xout = h->X1;
    f1.bias_out = L.b1; f1.g16 = h->G;
    rc |= launch_gemm_dec_ln<EPI_GELU16>(h, f1, s);
    DecGemmArgs f2{};
    f2.B = B; f2.Wp = L.w2; f2.N = d; f2.K = f; f2.a16 = h->G; f2.rout = h->r_f2;
    if (l + 1 < c.n_layers) {
      // the next layer's QKV GEMM comes next: its weights, b2 and ln2 scale / shift of this layer (contiguous
      // from b2 to ln2_b), and the bqkv that the attention after it starts with
      f2.pf = prefetch_for(h, h->layers[l + 1].wqkv, 3 * d, d, B);
      if (f2.pf.ptr) {
        set_aux(f2.pf, 0, L.b2, L.ln2_b + d);
        set_aux(f2.pf, 1, h->layers[l + 1].bqkv, h->layers[l + 1].bqkv + 3 * d);
      }
    }
    rc |= launch_gemm_dec<EPI_RAW>(h, f2, h->sk_f2, s);
  }
  const LayerPtrs& P = h->layers[c.n_layers - 1];
  { ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0); ROW_DISPATCH(d, hipLaunchKernelGGL(ln_partials_kernel<RC>, dim3(B), dim3(64), 0, s, h->r_f2, h->sk_f2, P.b2, h->X1, B, d,
                     P.ln2_g, P.ln2_b, c.ln_eps, h->X, hidden_out)); }
  DecGemmArgs z{};
  z.B = B; z.Wp = h->tok_p; z.N = c.vocab_kept; z.K = d; z.a16 = apply_head(h, h->X, B, s); z.logits_out = logits_out;
  z.bias_out = h->out_bias;
  z.strip_val = h->strip_val; z.strip_idx = h->strip_idx; z.strips = h->plan.strips;
  h->cand = h->plan.strips;
  {
    // the next step starts with layer 0's QKV GEMM on the embedding rows: its weights and the embedding
    // LayerNorm's scale / shift (contiguous) ride along with the projection
    z.pf = prefetch_for(h, h->layers[0].wqkv, 3 * d, d, B);
    if (z.pf.ptr) {
      set_aux(z.pf, 0, h->emb_g, h->emb_b + d);
      set_aux(z.pf, 1, h->layers[0].bqkv, h->layers[0].bqkv + 3 * d);
    }
  }
  rc |= launch_gemm_dec<EPI_ARGMAX>(h, z, 1, s);
  return rc ? ERNIE_EHIP : ERNIE_OK;
}

// The whole layer stack of a small-batch decode step as ONE persistent kernel (decode_persist.h), followed by
// the output projection.  Shapes it takes: whatever the small-batch path takes, FFN width up to 4096.
bool persist_decode_fits(const ErnieHandle* h, int B) {
  if (!(h->persist && h->xch && B <= h->plan.xch_batch && fused_decode_fits(h, B) && h->cfg.d_ffn <= 4096 && h->cu_count > 0))
    return false;
  // every GEMM phase is one unit per workgroup: (strips / strips per unit) x row groups <= workgroups
  const int d = h->cfg.d_model, f = h->cfg.d_ffn, rpw = B > 32 ? 2 : 1;
  const int zg = (B + 8 * rpw - 1) / (8 * rpw), zg5 = (B + 4 * rpw - 1) / (4 * rpw);
  const int units = std::max(std::max(((3 * d / 32 + 1) / 2) * zg, ((f / 32 + 1) / 2) * zg), (d / 32) * zg5);
  return units <= h->cu_count;
}

int decode_layers_persist(ErnieHandle* h, const int* tok, float* logits_out, float* hidden_out, hipStream_t s) {
  const ErnieConfig& c = h->cfg;
  const int B = h->B, d = c.d_model, f = c.d_ffn;
  PersistArgs a{};
  a.layers = h->ptab; a.n_layers = c.n_layers; a.B = B; a.d = d; a.f = f; a.H = c.n_heads; a.S = c.max_seq; a.eps = c.ln_eps;
  a.tok = tok; a.cache_len = h->lens; a.tok_emb = h->tok_rm; a.pos_emb = h->pos;
  a.seg_row = h->type_emb ? h->type_emb + d : nullptr; a.emb_g = h->emb_g; a.emb_b = h->emb_b;
  a.max_pos = c.max_pos; a.vocab_kept = c.vocab_kept; a.eos = h->eos; a.finished = h->finished;
  a.slot = h->compacted ? h->slot : nullptr;
  a.xch = h->xch; a.xo = h->plan.xo; a.epoch = h->epoch; a.X = h->X; a.hidden_out = hidden_out;
  a.dbg = h->persist_dbg;
  a.trace = (h->persist_trace && h->cu_count <= kPersistTraceGroups)
                ? reinterpret_cast<unsigned long long*>(h->arena + h->plan.trace) : nullptr;
  a.table_p = h->tok_p; a.table_strips = c.vocab_kept / 32;      // whole strips only
  a.err = h->err_host; a.spin_limit = h->persist_spin; a.stall = h->persist_stall; a.attn_nt = h->attn_nt;
  const int rpw = B > 32 ? 2 : 1;
  // dynamic LDS: the largest A tile ([8 or 16 rows][d + 8], [4 or 8 rows][f + 8] fp16), then the cross-wave
  // reduction buffer [8 waves][2 strips x 4 or 8 registers][64 lanes] fp32
  const size_t lds_a = (size_t)8 * rpw * (d + 8) * 2, lds_5 = (size_t)4 * rpw * (f + 8) * 2, lds_r = (size_t)8 * 2 * 4 * rpw * 256;
  const size_t red_off = (std::max(lds_a, lds_5) + 255) / 256 * 256;
  const size_t lds = red_off + lds_r;
  a.red_off = (unsigned)red_off;
  {
    // workgroups past the largest phase (rounded up to a multiple of 8, so that ids congruent mod 8 keep their
    // XCD) own no unit: they warm the L2 for the others.  The attention may take several rounds of the grid.
    const int zg = (B + 8 * rpw - 1) / (8 * rpw), zg5 = (B + 4 * rpw - 1) / (4 * rpw);
    int busy = std::max(std::max(((3 * d / 32 + 1) / 2) * zg, ((f / 32 + 1) / 2) * zg), (d / 32) * zg5);
    busy = std::max(busy, std::min((B * c.n_heads + 1) / 2, h->cu_count * 3 / 4));
    busy = (busy + 7) / 8 * 8;
    a.helpers_from = (h->persist_helpers && h->cu_count % 8 == 0 && h->cu_count - busy >= 8) ? busy : h->cu_count;
    a.kv_rows = std::min(c.max_seq, h->max_len + h->steps + 1);
  }
  if (lds > kPersistMaxLds) return ERNIE_EINVAL;
  {
    const double w_bytes = (double)c.n_layers * (4.0 * d * d + 2.0 * d * f) * 2.0;
    const double kv_bytes = (double)c.n_layers * 2.0 * (h->sum_len + (double)B * (h->steps + 1)) * d * 2.0;
    ProfScope prof(h, ERNIE_PROF_DEC_PERSIST, s, w_bytes + kv_bytes, 2.0 * B * (4.0 * d * d + 2.0 * d * f) * c.n_layers);
    const dim3 grid(h->cu_count), block(kPersistThreads);
    // attention: the first batch of cache rows, requested before q, k, v arrive, covers 192 keys (six groups per
    // wave); a longer cache is streamed in further batches
    // fragment registers per wave: one per 128 of the contraction (6 for the 768-wide model, else 8; the FFN
    // width in steps of 1024)
#define PERSIST_LAUNCH(RPW, FRD, FR5) hipLaunchKernelGGL((decode_persist_kernel<RPW, FRD, FR5, 6>), grid, block, lds, s, a)
#define PERSIST_BY_F(RPW) do { if (d <= 768 && f > 2048 && f <= 3072) PERSIST_LAUNCH(RPW, 6, 24); else if (f <= 1024) PERSIST_LAUNCH(RPW, 8, 8); \
                               else if (f <= 2048) PERSIST_LAUNCH(RPW, 8, 16); else if (f <= 3072) PERSIST_LAUNCH(RPW, 8, 24); \
                               else PERSIST_LAUNCH(RPW, 8, 32); } while (0)
    if (rpw == 1) PERSIST_BY_F(1); else PERSIST_BY_F(2);
#undef PERSIST_BY_F
#undef PERSIST_LAUNCH
  }
  DecGemmArgs z{};
  z.B = B; z.Wp = h->tok_p; z.N = c.vocab_kept; z.K = d; z.a16 = apply_head(h, h->X, B, s); z.logits_out = logits_out;
  z.bias_out = h->out_bias;
  z.strip_val = h->strip_val; z.strip_idx = h->strip_idx; z.strips = h->plan.strips;
  h->cand = h->plan.strips;
  return launch_gemm_dec<EPI_ARGMAX>(h, z, 1, s);
}

// Decode projections at B > 64: the batch is a real M dimension, so they run on the MFMA GEMM pipeline
// (64 x 64 tiles, BK = 64: measured 10-20 % faster than 128 x 64 at these shapes) with the contraction split
// over gridDim.y until at least 144 workgroups stream the weights, each keeping a slice of at least 192;
// partial results are fp32 [split][B][N].  Every further split adds a partial buffer that is written and read
// back: measured, 144 unsplit workgroups beat 288 split ones (QKV at B = 256: step -1.2 %) and 192 beat 384,
// while 128 lose to 256.
using SplitPipe = GemmPipe<2, 2, 1, 1, 64, 3>;

int pick_gemm_split(int B, int N, int K) {
  const long tiles = (long)((B + SplitPipe::kBM - 1) / SplitPipe::kBM) * ((N + SplitPipe::kBN - 1) / SplitPipe::kBN);
  int best = 1;
  for (int sk = 1; sk <= kBigMaxSplitK; sk *= 2) {
    if ((K / 64) % sk != 0 || (sk > 1 && K / sk < 192)) break;
    best = sk;
    if (tiles * sk >= 144) break;
  }
  return best;
}

void launch_gemm_splitk(ErnieHandle* h, const half_t* A, const half_t* Wp, int M, int N, int K, float* out, int sk,
                        hipStream_t s) {
  ProfScope prof(h, ERNIE_PROF_GEMM_DEC, s, 2.0 * N * K, 2.0 * M * N * K);
  using P = SplitPipe;
  const int tiles_m = (M + P::kBM - 1) / P::kBM, tiles_n = (N + P::kBN - 1) / P::kBN;
  if (h->big_narrow && (long)tiles_m * tiles_n * sk * 2 <= 256) {
    // too few 64 x 64 tiles for the CUs even after the split of the contraction: 64 x 32 tiles double them
    using Q = GemmPipe<2, 1, 1, 1, 64, 3>;
    const int tn = (N + Q::kBN - 1) / Q::kBN;
    hipLaunchKernelGGL((gemm_prefill2_kernel<2, 1, 1, 1, 64, 3, EpiRaw32>), dim3(tiles_m * tn, sk), dim3(128),
                       Q::kLdsBytes, s, A, Wp, h->zero_bias, M, N, K, (N + 31) / 32, (h->big_mfast && tiles_m == 2) ? -tiles_m : tn,
                       EpiRaw32{out, N, (size_t)M * N});
    return;
  }
  hipLaunchKernelGGL((gemm_prefill2_kernel<2, 2, 1, 1, 64, 3, EpiRaw32>), dim3(tiles_m * tiles_n, sk), dim3(256),
                     P::kLdsBytes, s, A, Wp, h->zero_bias, M, N, K, (N + 31) / 32, (h->big_mfast && tiles_m == 2) ? -tiles_m : tiles_n,
                     EpiRaw32{out, N, (size_t)M * N});
}

// Output projection at B > 64 on the MFMA GEMM pipeline: fp32 partial logits (one or two splits of the
// contraction), then one workgroup per sequence adds them and takes the row argmax.
void launch_logits_big(ErnieHandle* h, const half_t* X, int B, float* logits_out, hipStream_t s) {
  using P = SplitPipe;
  const int N = h->cfg.vocab_kept, K = h->cfg.d_model;
  const int tiles_m = (B + P::kBM - 1) / P::kBM, tiles_n = (N + P::kBN - 1) / P::kBN;
  const int sk = (tiles_m * tiles_n < 144 && (K / 64) % 2 == 0 && K / 2 >= 192) ? 2 : 1;
  hipLaunchKernelGGL((gemm_prefill2_kernel<2, 2, 1, 1, 64, 3, EpiRaw32>), dim3(tiles_m * tiles_n, sk), dim3(256),
                     P::kLdsBytes, s, X, h->tok_p, h->zero_bias, B, N, K, (N + 31) / 32, tiles_n,
                     EpiRaw32{h->r_logits, N, (size_t)B * N});
  hipLaunchKernelGGL(logits_rows_argmax_kernel, dim3(B), dim3(256), 0, s, h->r_logits, sk, B, N, h->out_bias, logits_out,
                     h->strip_val, h->strip_idx);
}

// Optional output head: t = LayerNorm(gelu(head_w x + head_b)) for the B final rows `x`, written to hlast
// (x may be hlast itself: the GEMM has consumed it before the row kernel overwrites it).  Returns the rows
// the tied projection reads.
const half_t* apply_head(ErnieHandle* h, const half_t* x, int B, hipStream_t s) {
  if (!h->head_w) return x;
  const int d = h->cfg.d_model;
  const int sk = pick_gemm_split(B, d, d);
  launch_gemm_splitk(h, x, h->head_w, B, d, d, h->r_out, sk, s);
  ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0);
  ROW_DISPATCH(d, hipLaunchKernelGGL((ln_partials_kernel<RC, true>), dim3(B), dim3(64), 0, s, h->r_out, sk,
                                     h->head_b, (const half_t*)nullptr, B, d, h->head_g, h->head_beta, h->cfg.ln_eps,
                                     h->hlast, (float*)nullptr));
  return h->hlast;
}

// Larger batches (B > 64): split-K MFMA GEMMs write fp32 partials; the attention prologue and two row
// kernels add partials + bias (+ residual) and apply LayerNorm; FFN1 keeps its contraction whole with bias +
// GELU in its epilogue.  7 launches per layer; the cache stream of the attention is the largest share of the step.
int decode_layers_big(ErnieHandle* h, float* logits_out, float* hidden_out, hipStream_t s) {
  const ErnieConfig& c = h->cfg;
  const int B = h->B, d = c.d_model, f = c.d_ffn;
  const int sk_q = pick_gemm_split(B, 3 * d, d), sk_o = pick_gemm_split(B, d, d), sk_1 = pick_gemm_split(B, f, d),
            sk_2 = pick_gemm_split(B, d, f);
  const int rpw = h->big_ln_rows;        // rows per workgroup of the LayerNorm row kernels
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerPtrs& L = h->layers[l];
    launch_gemm_splitk(h, h->X, L.wqkv, B, 3 * d, d, h->r_qkv, sk_q, s);
    {
      ProfScope prof(h, ERNIE_PROF_ATTN_DEC, s, 2.0 * (h->sum_len + (double)B * (h->steps + 1)) * d * 2.0, 0.0);
      // the attention is the long kernel of the step: a few extra workgroups pull the small vectors that the
      // row kernels and the FFN1 epilogue of this layer (bo .. ln2_b, contiguous) and the next attention
      // (its bqkv) start with into every XCD's L2
      DecPrefetch warm{};
      if (h->big_warm > 0) {
        warm.count = h->big_warm;
        set_aux(warm, 0, L.bo, L.ln2_b + d);
        if (l + 1 < c.n_layers) set_aux(warm, 1, h->layers[l + 1].bqkv, h->layers[l + 1].bqkv + 3 * d);
      }
      launch_attn_decode(h, h->r_qkv, sk_q, B, L.bqkv, kcache(h, l), vcache(h, l), s, warm);
    }
    launch_gemm_splitk(h, h->O, L.wo, B, d, d, h->r_out, sk_o, s);
    { ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0);
      ROW_DISPATCH(d, hipLaunchKernelGGL(ln_partials_kernel<RC>, dim3((B + rpw - 1) / rpw), dim3(64 * rpw), 0, s, h->r_out, sk_o,
                                         L.bo, h->X, B, d, L.ln1_g, L.ln1_b, c.ln_eps, h->X1, (float*)nullptr)); }
    if (h->big_f1_fused) {
      // FFN1 keeps its contraction whole: bias + GELU in the GEMM epilogue, no partial buffers and one launch
      // less (the wide N gives enough 64 x 64 tiles; the unsplit GEMM costs 0.3-1.6 us more, a launch 5-6 us)
      ProfScope prof(h, ERNIE_PROF_GEMM_DEC, s, 2.0 * f * d, 2.0 * B * f * d);
      // 64 x 32 tiles when 64 x 64 ones would leave half the CUs without a workgroup (measured +0.5 % at
      // B = 128, f = 4096; -0.6 % at B = 256, f = 3072, where 64 x 64 already gives 192 workgroups)
      const long tiles64 = (long)((B + 63) / 64) * ((f + 63) / 64);
      const bool narrow = h->big_f1_tile == 1 || (h->big_f1_tile == 0 && tiles64 * 2 <= 256);
      // the narrow tile's stages are 12 KB, so its ring is five deep (16 k-steps, unsplit: -1.1 % of the step at
      // B = 128); five stages of the 64 x 64 tile, or of the split projections, measured slower
      if (narrow) launch_gemm_prefill_t<2, 1, 1, 1, 64, 5>(h->X1, L.w1, L.b1, B, f, d, EpiGeluFast{h->G, f}, s, h->big_mfast && (B + 63) / 64 == 2);
      else launch_gemm_prefill_t<2, 2, 1, 1, 64, 3>(h->X1, L.w1, L.b1, B, f, d, EpiGeluFast{h->G, f}, s, h->big_mfast && (B + 63) / 64 == 2);
    } else {
      launch_gemm_splitk(h, h->X1, L.w1, B, f, d, h->r_f1, sk_1, s);
      ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0);
      const size_t n8 = (size_t)B * f / 8;
      hipLaunchKernelGGL(gelu_partials_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, h->r_f1, sk_1, L.b1,
                         B, f, h->G);
    }
    launch_gemm_splitk(h, h->G, L.w2, B, d, f, h->r_f2, sk_2, s);
    { ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0);
      float* hid = (l == c.n_layers - 1) ? hidden_out : nullptr;
      ROW_DISPATCH(d, hipLaunchKernelGGL(ln_partials_kernel<RC>, dim3((B + rpw - 1) / rpw), dim3(64 * rpw), 0, s, h->r_f2, sk_2,
                                         L.b2, h->X1, B, d, L.ln2_g, L.ln2_b, c.ln_eps, h->X, hid)); }
  }
  const half_t* x = apply_head(h, h->X, B, s);
  { ProfScope prof(h, ERNIE_PROF_LOGITS, s, 2.0 * c.vocab_kept * d, 2.0 * B * c.vocab_kept * d);
    h->cand = launch_logits(h, x, B, logits_out, s); }
  return ERNIE_OK;
}

void pack_into(const void* src, half_t* dst, int N, int K, hipStream_t s) {
  const int n_tiles = (N + 31) / 32;
  const size_t total = (size_t)n_tiles * (K / 16) * 64;
  const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
  hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks), dim3(256), 0, s, (const half_t*)src, dst, N, K, n_tiles);
}

void cvt_into(const void* src, float* dst, int n, hipStream_t s) {
  hipLaunchKernelGGL(cvt_f16_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, (const half_t*)src, dst, n);
}

}  // namespace

extern "C" {

const char* ernie_error_string(int code) {
  switch (code) {
    case ERNIE_OK: return "ok";
    case ERNIE_EINVAL: return "invalid argument";
    case ERNIE_ECAPACITY: return "capacity exceeded (batch, sequence or position)";
    case ERNIE_EARENA: return "arena too small";
    case ERNIE_ESEQUENCE: return "decode step before prefill";
    case ERNIE_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

int ernie_init_weights(const ErnieConfig* cfg, const ErnieWeights* w, void* arena_dev, size_t arena_bytes,
                       size_t* arena_needed, void* stream, ErnieHandle** out) {
  return ernie_init_weights_ex(cfg, w, nullptr, arena_dev, arena_bytes, arena_needed, stream, out);
}

int ernie_init_weights_ex(const ErnieConfig* cfg, const ErnieWeights* w, const ErnieVariants* var, void* arena_dev,
                          size_t arena_bytes, size_t* arena_needed, void* stream, ErnieHandle** out) {
  const int rc = check_config(cfg);
  if (rc != ERNIE_OK) return rc;
  if (var) {
    const int n_head = (var->head_w != nullptr) + (var->head_b != nullptr) + (var->head_ln_g != nullptr) +
                       (var->head_ln_b != nullptr);
    if (n_head != 0 && n_head != 4) return ERNIE_EINVAL;
  }
  ArenaPlan plan = make_plan(*cfg, var);
  if (arena_needed) *arena_needed = plan.total;
  if (!arena_dev) return arena_needed ? ERNIE_OK : ERNIE_EINVAL;
  if (!w || !out) return ERNIE_EINVAL;
  if ((uintptr_t)arena_dev % kAlign != 0) return ERNIE_EINVAL;
  if (arena_bytes < plan.total) return ERNIE_EARENA;
  if (!w->tok_emb_kept || !w->kept_ids || !w->pos_emb || !w->emb_ln_g || !w->emb_ln_b || !w->wqkv || !w->bqkv ||
      !w->wo || !w->bo || !w->ln1_g || !w->ln1_b || !w->w1 || !w->b1 || !w->w2 || !w->b2 || !w->ln2_g || !w->ln2_b)
    return ERNIE_EINVAL;
  for (int l = 0; l < cfg->n_layers; ++l)
    if (!w->wqkv[l] || !w->bqkv[l] || !w->wo[l] || !w->bo[l] || !w->ln1_g[l] || !w->ln1_b[l] || !w->w1[l] ||
        !w->b1[l] || !w->w2[l] || !w->b2[l] || !w->ln2_g[l] || !w->ln2_b[l])
      return ERNIE_EINVAL;

  ErnieHandle* h = new (std::nothrow) ErnieHandle();
  if (!h) return ERNIE_EHIP;
  h->cfg = *cfg;
  h->plan = plan;
  unsigned char* a = static_cast<unsigned char*>(arena_dev);
  h->arena = a;
  auto H16 = [&](size_t o) { return reinterpret_cast<half_t*>(a + o); };
  auto F32 = [&](size_t o) { return reinterpret_cast<float*>(a + o); };
  auto I32 = [&](size_t o) { return reinterpret_cast<int*>(a + o); };
  h->tok_rm = H16(plan.tok_rm); h->tok_p = H16(plan.tok_p); h->pos = H16(plan.pos);
  h->emb_g = F32(plan.emb_g); h->emb_b = F32(plan.emb_b);
  h->kv = H16(plan.kv); h->X = H16(plan.X); h->X1 = H16(plan.X1); h->Y = H16(plan.Y); h->Q = H16(plan.Q);
  h->O = H16(plan.O); h->G = H16(plan.G); h->hlast = H16(plan.hlast);
  h->Yf = F32(plan.Yf); h->strip_val = F32(plan.strip_val);
  h->r_qkv = F32(plan.r_qkv); h->r_out = F32(plan.r_out); h->r_f1 = F32(plan.r_f1); h->r_f2 = F32(plan.r_f2); h->zero_bias = F32(plan.zero_bias);
  h->fused_decode = 1;
  h->attn_dec = 0;
  h->sk_out = pick_split_k(cfg->d_model / 32, cfg->d_model / 16, 2);
  h->sk_f2 = pick_split_k(cfg->d_model / 32, cfg->d_ffn / 16, 4);
  h->strip_idx = I32(plan.strip_idx); h->cu = I32(plan.cu); h->lens = I32(plan.lens);
  h->tok_seq = I32(plan.tok_seq); h->tok_pos = I32(plan.tok_pos); h->tok_prev = I32(plan.tok_prev);
  h->finished = I32(plan.finished); h->slot = I32(plan.slot); h->keep = I32(plan.keep);
  h->r_logits = F32(plan.r_logits);
  if (plan.xch_batch > 0) {
    h->xch = a + plan.xch; h->ptab = reinterpret_cast<PersistLayer*>(a + plan.ptab);
    h->epoch = reinterpret_cast<unsigned*>(a + plan.epoch);
  }
  h->prefilled = false; h->B = 0; h->max_len = 0; h->steps = 0; h->sum_len = h->sum_len2 = 0.0;
  h->staging = nullptr; h->staging_next = 0; h->staging_captured = 0;
  for (int i = 0; i < kStagingSlots; ++i) { h->stage_ev[i] = nullptr; h->stage_busy[i] = false; }

  hipStream_t s = static_cast<hipStream_t>(stream);
  bool host_ok = configure_kernels() == ERNIE_OK && static_scratch_for_current_device(&h->static_scratch) == ERNIE_OK &&
                 hipHostMalloc(reinterpret_cast<void**>(&h->staging),
                               sizeof(int) * (2 * kStagingSlots * (cfg->max_batch + 1) + 16), hipHostMallocDefault) == hipSuccess;
  if (host_ok) {
    h->err_host = h->staging + (size_t)2 * kStagingSlots * (cfg->max_batch + 1);     // behind the staging slots
    *h->err_host = 0;
    int dev = 0;
    host_ok = hipGetDevice(&dev) == hipSuccess &&
              hipDeviceGetAttribute(&h->cu_count, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess;
  }
  for (int i = 0; host_ok && i < kStagingSlots; ++i)
    host_ok = hipEventCreateWithFlags(&h->stage_ev[i], hipEventDisableTiming) == hipSuccess;
  if (!host_ok) {
    ernie_free(h);
    return ERNIE_EHIP;
  }

  const int d = cfg->d_model, f = cfg->d_ffn, V = cfg->vocab_kept;
  bool copies_ok = true;
  copies_ok &= hipMemsetAsync(h->zero_bias, 0, (size_t)std::max(std::max(3 * d, f), V) * 4, s) == hipSuccess;
  copies_ok &= hipMemcpyAsync(h->tok_rm, w->tok_emb_kept, (size_t)V * d * 2, hipMemcpyDeviceToDevice, s) == hipSuccess;
  copies_ok &= hipMemcpyAsync(h->pos, w->pos_emb, (size_t)cfg->max_pos * d * 2, hipMemcpyDeviceToDevice, s) == hipSuccess;
  copies_ok &= hipMemcpyAsync(a + plan.kept, w->kept_ids, (size_t)V * 4, hipMemcpyDeviceToDevice, s) == hipSuccess;
  pack_into(w->tok_emb_kept, h->tok_p, V, d, s);
  cvt_into(w->emb_ln_g, h->emb_g, d, s);
  cvt_into(w->emb_ln_b, h->emb_b, d, s);
  h->layers.resize(cfg->n_layers);
  for (int l = 0; l < cfg->n_layers; ++l) {
    const ArenaPlan::L& o = plan.layers[l];
    LayerPtrs& L = h->layers[l];
    L.wqkv = H16(o.wqkv); L.wo = H16(o.wo); L.w1 = H16(o.w1); L.w2 = H16(o.w2);
    L.bqkv = F32(o.bqkv); L.bo = F32(o.bo); L.b1 = F32(o.b1); L.b2 = F32(o.b2);
    L.ln1_g = F32(o.ln1_g); L.ln1_b = F32(o.ln1_b); L.ln2_g = F32(o.ln2_g); L.ln2_b = F32(o.ln2_b);
    pack_into(w->wqkv[l], L.wqkv, 3 * d, d, s);
    pack_into(w->wo[l], L.wo, d, d, s);
    pack_into(w->w1[l], L.w1, f, d, s);
    pack_into(w->w2[l], L.w2, d, f, s);
    cvt_into(w->bqkv[l], L.bqkv, 3 * d, s); cvt_into(w->bo[l], L.bo, d, s);
    cvt_into(w->b1[l], L.b1, f, s); cvt_into(w->b2[l], L.b2, d, s);
    cvt_into(w->ln1_g[l], L.ln1_g, d, s); cvt_into(w->ln1_b[l], L.ln1_b, d, s);
    cvt_into(w->ln2_g[l], L.ln2_g, d, s); cvt_into(w->ln2_b[l], L.ln2_b, d, s);
  }
  if (h->xch) {
    // tags start at zero everywhere, so that the first step's tag (1) is new to every pair
    copies_ok &= hipMemsetAsync(h->xch, 0, (size_t)plan.xo.layer_bytes * cfg->n_layers, s) == hipSuccess;
    copies_ok &= hipMemsetAsync(h->epoch, 0, 256, s) == hipSuccess;
    copies_ok &= hipMemsetAsync(a + plan.trace, 0, (size_t)kPersistTraceGroups * cfg->n_layers * 32 * 8, s) == hipSuccess;
    h->ptab_host.resize(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
      const LayerPtrs& L = h->layers[l];
      h->ptab_host[l] = PersistLayer{L.wqkv, L.wo, L.w1, L.w2, L.bqkv, L.bo, L.b1, L.b2, L.ln1_g, L.ln1_b, L.ln2_g,
                                     L.ln2_b, kcache(h, l), vcache(h, l)};
    }
    copies_ok &= hipMemcpyAsync(h->ptab, h->ptab_host.data(), sizeof(PersistLayer) * cfg->n_layers,
                                hipMemcpyHostToDevice, s) == hipSuccess;
  }
  if (plan.has_type) {
    h->type_emb = H16(plan.type_emb);
    copies_ok &= hipMemcpyAsync(h->type_emb, var->type_emb, (size_t)2 * d * 2, hipMemcpyDeviceToDevice, s) == hipSuccess;
  }
  if (plan.has_head) {
    h->head_w = H16(plan.head_w); h->head_b = F32(plan.head_b); h->head_g = F32(plan.head_g);
    h->head_beta = F32(plan.head_beta);
    pack_into(var->head_w, h->head_w, d, d, s);
    cvt_into(var->head_b, h->head_b, d, s); cvt_into(var->head_ln_g, h->head_g, d, s);
    cvt_into(var->head_ln_b, h->head_beta, d, s);
  }
  if (plan.has_bias) {
    h->out_bias = F32(plan.out_bias);
    cvt_into(var->out_bias, h->out_bias, V, s);
  }
  if (launch_status() != ERNIE_OK || !copies_ok) {
    ernie_free(h);
    return ERNIE_EHIP;
  }
  *out = h;
  return ERNIE_OK;
}

int ernie_prefill(ErnieHandle* h, int32_t B, int32_t Lmax, const int32_t* ids_dev, const int32_t* prompt_lens_host,
                  float* logits_out_dev, float* hidden_out_dev, int32_t* tok_out_dev, void* stream) {
  if (!h || !ids_dev || !prompt_lens_host || !tok_out_dev) return ERNIE_EINVAL;
  if (B < 1 || Lmax < 1) return ERNIE_EINVAL;
  const ErnieConfig& c = h->cfg;
  if (B > c.max_batch || Lmax > c.max_seq || Lmax > c.max_pos) return ERNIE_ECAPACITY;
  int max_len = 0;
  double sum_len = 0.0, sum_len2 = 0.0;
  for (int b = 0; b < B; ++b) {
    const int L = prompt_lens_host[b];
    if (L < 1 || L > Lmax) return ERNIE_EINVAL;
    if (L > max_len) max_len = L;
    sum_len += L; sum_len2 += (double)L * L;
  }

  hipStream_t s = static_cast<hipStream_t>(stream);
  int stage_slot;
  int* stage = stage_acquire(h, s, &stage_slot);
  if (!stage) return ERNIE_ECAPACITY;
  stage[0] = 0;
  for (int b = 0; b < B; ++b) stage[b + 1] = stage[b] + prompt_lens_host[b];
  const int T = stage[B];
  HIP_OK(hipMemcpyAsync(h->cu, stage, sizeof(int) * (B + 1), hipMemcpyHostToDevice, s));
  stage_release(h, s, stage_slot);

  const int d = c.d_model, f = c.d_ffn, H = c.n_heads, S = c.max_seq;
  { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0); hipLaunchKernelGGL(token_map_kernel, dim3((T + 255) / 256), dim3(256), 0, s, h->cu, B, T, h->tok_seq, h->tok_pos,
                     h->lens, h->finished, h->slot); }
  { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0); ROW_DISPATCH(d, hipLaunchKernelGGL(embed_ln_prefill_kernel<RC>, dim3((T + 3) / 4), dim3(256), 0, s, ids_dev, Lmax, h->tok_seq,
                     h->tok_pos, T, h->tok_rm, h->pos, h->type_emb, h->emb_g, h->emb_b, c.ln_eps, d, h->X, c.vocab_kept)); }
  const int q_tiles = (max_len + kAttnQTile - 1) / kAttnQTile;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerPtrs& L = h->layers[l];
    EpiQKV eq{h->Q, kcache(h, l), vcache(h, l), h->tok_seq, h->tok_pos, d, H, S, T};
    launch_gemm_prefill(h, h->X, L.wqkv, L.bqkv, T, 3 * d, d, eq, s);
    {
      ProfScope prof(h, ERNIE_PROF_ATTN_PREFILL, s, 0.0, 4.0 * sum_len2 * d);
      hipLaunchKernelGGL(attn_prefill_kernel, dim3(q_tiles, H, B), dim3(256), kAttnLdsBytes, s, h->Q, kcache(h, l), vcache(h, l),
                         h->cu, T, H, S, d, h->O);
    }
    launch_gemm_prefill(h, h->O, L.wo, L.bo, T, d, d, EpiResidual{h->X, h->Y, d}, s);
    { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0); ROW_DISPATCH(d, hipLaunchKernelGGL(ln_rows_f16_kernel<RC>, dim3((T + 3) / 4), dim3(256), 0, s, h->Y, T, d, L.ln1_g, L.ln1_b, c.ln_eps,
                       h->X1)); }
    launch_gemm_prefill(h, h->X1, L.w1, L.b1, T, f, d, EpiGelu{h->G, f}, s);
    launch_gemm_prefill(h, h->G, L.w2, L.b2, T, d, f, EpiResidual{h->X1, h->Y, d}, s);
    { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0); ROW_DISPATCH(d, hipLaunchKernelGGL(ln_rows_f16_kernel<RC>, dim3((T + 3) / 4), dim3(256), 0, s, h->Y, T, d, L.ln2_g, L.ln2_b, c.ln_eps,
                       h->X)); }
  }
  { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0); hipLaunchKernelGGL(gather_last_rows_kernel, dim3(B), dim3(256), 0, s, h->X, h->cu, B, d, h->hlast, hidden_out_dev); }
  const half_t* xhead = apply_head(h, h->hlast, B, s);
  { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0);
  h->cand = launch_logits(h, xhead, B, logits_out_dev, s);
  }
  { ProfScope prof(h, ERNIE_PROF_ROW_PREFILL, s, 0.0, 0.0);
  hipLaunchKernelGGL(argmax_final_kernel, dim3(B), dim3(256), 0, s, h->strip_val, h->strip_idx, h->cand,
                     tok_out_dev, h->tok_prev, h->lens, 0, S, c.vocab_kept, (const int*)nullptr, -1);
  }
  h->compacted = false;
  h->row_len.assign(prompt_lens_host, prompt_lens_host + B);
  h->prefilled = true; h->B = B; h->max_len = max_len; h->steps = 0;
  h->sum_len = sum_len; h->sum_len2 = sum_len2;
  return launch_status();
}

// Host-side checks shared by the two decode entry points.
static int decode_step_checks(const ErnieHandle* h, const int32_t* tok_out_dev) {
  if (!h || !tok_out_dev) return ERNIE_EINVAL;
  if (!h->prefilled) return ERNIE_ESEQUENCE;
  // a bounded wait of the one-launch decode kernel gave up in an earlier step: reported once, here
  if (h->err_host && *(volatile int*)h->err_host) { *(volatile int*)h->err_host = 0; return ERNIE_EHIP; }
  const ErnieConfig& c = h->cfg;
  const int next_pos = h->max_len + h->steps;          // position / cache slot of the longest sequence's new token
  if (next_pos + 1 > c.max_seq || next_pos >= c.max_pos) return ERNIE_ECAPACITY;
  return ERNIE_OK;
}

static int decode_step_enqueue(ErnieHandle* h, const int32_t* tok_in_dev, float* logits_out_dev, float* hidden_out_dev,
                               int32_t* tok_out_dev, void* stream) {
  const ErnieConfig& c = h->cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = h->B, d = c.d_model;
  const int* tok = tok_in_dev ? tok_in_dev : h->tok_prev;
  int rc;
  if (persist_decode_fits(h, B)) {
    rc = decode_layers_persist(h, tok, logits_out_dev, hidden_out_dev, s);
  } else if (fused_decode_fits(h, B)) {
    rc = decode_layers_fused(h, tok, logits_out_dev, hidden_out_dev, s);
  } else {
    { ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0); ROW_DISPATCH(d, hipLaunchKernelGGL(embed_ln_decode_kernel<RC>, dim3(B), dim3(64), 0, s, tok, h->lens, B, c.max_pos,
                       h->tok_rm, h->pos, h->type_emb ? h->type_emb + d : nullptr, h->emb_g, h->emb_b, c.ln_eps, d, h->X,
                       h->eos, h->finished, c.vocab_kept)); }
    rc = decode_layers_big(h, logits_out_dev, hidden_out_dev, s);
  }
  if (rc != ERNIE_OK) return rc;
  { ProfScope prof(h, ERNIE_PROF_ROW_DEC, s, 0.0, 0.0);
  hipLaunchKernelGGL(argmax_final_kernel, dim3(B), dim3(256), 0, s, h->strip_val, h->strip_idx, h->cand,
                     tok_out_dev, h->tok_prev, h->lens, 1, c.max_seq, c.vocab_kept,
                     h->eos >= 0 ? h->finished : (const int*)nullptr, h->eos, h->epoch);
  }
  h->steps += 1;
  return launch_status();
}

int ernie_decode_step(ErnieHandle* h, const int32_t* tok_in_dev, float* logits_out_dev, float* hidden_out_dev,
                      int32_t* tok_out_dev, void* stream) {
  const int rc = decode_step_checks(h, tok_out_dev);
  if (rc != ERNIE_OK) return rc;
  return decode_step_enqueue(h, tok_in_dev, logits_out_dev, hidden_out_dev, tok_out_dev, stream);
}

int ernie_decode_step_static(ErnieHandle* h, const int32_t* tok_in_dev, float* logits_out_dev, float* hidden_out_dev,
                             int32_t* tok_out_dev, void* stream) {
  const int rc = decode_step_checks(h, tok_out_dev);
  if (rc != ERNIE_OK) return rc;
  const ErnieConfig& c = h->cfg;
  // sizes beyond the static array's layout are refused before anything is enqueued
  if (!h->static_scratch) return ERNIE_EHIP;
  if (h->B > kStaticMaxBatch || c.d_model > kStaticMaxWidth || c.d_ffn > kStaticMaxFfn ||
      h->plan.strips > kStaticMaxStrips || h->sk_f2 > 4 || !fused_decode_fits(h, h->B))
    return ERNIE_ECAPACITY;
  // the step's temporaries move from the arena to the static array for this call; weights, the key/value
  // cache and the per-sequence state stay where they are
  struct Saved { float *r_qkv, *r_out, *r_f2, *strip_val; int* strip_idx; half_t *X, *X1, *O, *G, *hlast; };
  const Saved keep{h->r_qkv, h->r_out, h->r_f2, h->strip_val, h->strip_idx, h->X, h->X1, h->O, h->G, h->hlast};
  unsigned char* base = h->static_scratch;
  h->r_qkv = reinterpret_cast<float*>(base + StaticLayout::r_qkv);
  h->r_out = reinterpret_cast<float*>(base + StaticLayout::r_out);
  h->r_f2 = reinterpret_cast<float*>(base + StaticLayout::r_f2);
  h->strip_val = reinterpret_cast<float*>(base + StaticLayout::strip_val);
  h->strip_idx = reinterpret_cast<int*>(base + StaticLayout::strip_idx);
  h->X = reinterpret_cast<half_t*>(base + StaticLayout::X);
  h->X1 = reinterpret_cast<half_t*>(base + StaticLayout::X1);
  h->O = reinterpret_cast<half_t*>(base + StaticLayout::O);
  h->hlast = reinterpret_cast<half_t*>(base + StaticLayout::hlast);
  h->G = reinterpret_cast<half_t*>(base + StaticLayout::G);
  const int persist_was = h->persist;
  h->persist = 0;                    // the one-launch kernel's exchange buffers are arena memory: not used here
  const int out = decode_step_enqueue(h, tok_in_dev, logits_out_dev, hidden_out_dev, tok_out_dev, stream);
  h->persist = persist_was;
  h->r_qkv = keep.r_qkv; h->r_out = keep.r_out; h->r_f2 = keep.r_f2; h->strip_val = keep.strip_val;
  h->strip_idx = keep.strip_idx; h->X = keep.X; h->X1 = keep.X1; h->O = keep.O; h->G = keep.G; h->hlast = keep.hlast;
  return out;
}

int ernie_last_error(ErnieHandle* h) {
  if (!h) return ERNIE_EINVAL;
  if (h->err_host && *(volatile int*)h->err_host) { *(volatile int*)h->err_host = 0; return ERNIE_EHIP; }
  return ERNIE_OK;
}

int ernie_get_config(const ErnieHandle* h, ErnieConfig* out) {
  if (!h || !out) return ERNIE_EINVAL;
  *out = h->cfg;
  return ERNIE_OK;
}

int ernie_set_eos(ErnieHandle* h, int32_t eos_id) {
  if (!h || eos_id < -1 || eos_id >= h->cfg.vocab_kept) return ERNIE_EINVAL;
  h->eos = eos_id;
  return ERNIE_OK;
}

int ernie_batch_state(ErnieHandle* h, int32_t* lens_out_dev, int32_t* finished_out_dev, void* stream) {
  if (!h) return ERNIE_EINVAL;
  if (!h->prefilled) return ERNIE_ESEQUENCE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int B = h->B;
  if (lens_out_dev) hipLaunchKernelGGL(copy_ints_kernel, dim3((B + 255) / 256), dim3(256), 0, s, h->lens, lens_out_dev, B);
  if (finished_out_dev)
    hipLaunchKernelGGL(copy_ints_kernel, dim3((B + 255) / 256), dim3(256), 0, s, h->finished, finished_out_dev, B);
  return launch_status();
}

int ernie_compact(ErnieHandle* h, int32_t n_keep, const int32_t* keep_rows_host, void* stream) {
  if (!h || !keep_rows_host) return ERNIE_EINVAL;
  if (!h->prefilled) return ERNIE_ESEQUENCE;
  if (n_keep < 1 || n_keep > h->B) return ERNIE_EINVAL;
  for (int i = 0; i < n_keep; ++i) {
    const int r = keep_rows_host[i];
    if (r < 0 || r >= h->B || (i > 0 && r <= keep_rows_host[i - 1])) return ERNIE_EINVAL;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool identity = true;
  for (int i = 0; i < n_keep; ++i) identity &= (keep_rows_host[i] == i);
  if (!identity) {
    int stage_slot;
    int* stage = stage_acquire(h, s, &stage_slot);
    if (!stage) return ERNIE_ECAPACITY;
    for (int i = 0; i < n_keep; ++i) stage[i] = keep_rows_host[i];
    HIP_OK(hipMemcpyAsync(h->keep, stage, sizeof(int) * n_keep, hipMemcpyHostToDevice, s));
    stage_release(h, s, stage_slot);
    hipLaunchKernelGGL(batch_compact_kernel, dim3(1), dim3(256), 0, s, h->keep, n_keep, h->lens, h->tok_prev,
                       h->finished, h->slot);
    h->compacted = true;
  }
  double sum_len = 0.0, sum_len2 = 0.0;
  for (int i = 0; i < n_keep; ++i) {
    const int L = h->row_len[keep_rows_host[i]];
    h->row_len[i] = L;
    sum_len += L; sum_len2 += (double)L * L;
  }
  h->row_len.resize(n_keep);
  h->sum_len = sum_len; h->sum_len2 = sum_len2;
  h->B = n_keep;
  return launch_status();
}

int ernie_plan_batches(const int32_t* lens_host, int32_t n, int32_t max_batch, int64_t max_tokens,
                       int32_t* order_out_host, int32_t* starts_out_host, int32_t* n_batches_out) {
  if (n < 0 || max_batch < 1 || max_tokens < 1 || !n_batches_out || !starts_out_host) return ERNIE_EINVAL;
  if (n > 0 && (!lens_host || !order_out_host)) return ERNIE_EINVAL;
  for (int i = 0; i < n; ++i)
    if (lens_host[i] < 1 || lens_host[i] > max_tokens) return ERNIE_EINVAL;
  for (int i = 0; i < n; ++i) order_out_host[i] = i;
  std::stable_sort(order_out_host, order_out_host + n,
                   [&](int32_t a, int32_t b) { return lens_host[a] < lens_host[b]; });
  int nb = 0;
  int64_t rows = 0;
  starts_out_host[0] = 0;
  for (int pos = 0; pos < n; ++pos) {
    const int64_t L = lens_host[order_out_host[pos]];     // ascending: the candidate is the longest of its batch
    if (rows + 1 > max_batch || (rows + 1) * L > max_tokens) {
      starts_out_host[++nb] = pos;
      rows = 0;
    }
    ++rows;
  }
  if (n > 0) starts_out_host[++nb] = n;
  *n_batches_out = nb;
  return ERNIE_OK;
}

void ernie_free(ErnieHandle* h) {
  if (!h) return;
  for (int i = 0; i < kStagingSlots; ++i) {
    if (h->stage_busy[i]) (void)hipEventSynchronize(h->stage_ev[i]);     // the copy still reads the pinned slot
    if (h->stage_ev[i]) (void)hipEventDestroy(h->stage_ev[i]);
  }
  if (h->staging) (void)hipHostFree(h->staging);
  for (auto& sl : h->prof.slots) { (void)hipEventDestroy(sl.a); (void)hipEventDestroy(sl.b); }
  delete h;
}

int ernie_debug_buffer(ErnieHandle* h, const char* name, void** ptr_dev, size_t* bytes) {
  if (!h || !name || !ptr_dev || !bytes) return ERNIE_EINVAL;
  const ErnieConfig& c = h->cfg;
  if (!strcmp(name, "x")) {
    *ptr_dev = h->X; *bytes = h->plan.t_max * c.d_model * 2;
  } else if (!strcmp(name, "kv")) {
    *ptr_dev = h->kv; *bytes = (size_t)c.n_layers * 2 * c.max_batch * c.max_seq * c.d_model * 2;
  } else if (!strcmp(name, "lens")) {
    *ptr_dev = h->lens; *bytes = (size_t)c.max_batch * 4;
  } else if (!strcmp(name, "persist_trace") && h->xch) {
    *ptr_dev = h->arena + h->plan.trace; *bytes = (size_t)h->cu_count * c.n_layers * 32 * 8;
  } else {
    return ERNIE_EINVAL;
  }
  return ERNIE_OK;
}

int ernie_profile(ErnieHandle* h, int enable) {
  if (!h) return ERNIE_EINVAL;
  Profiler& p = h->prof;
  if (enable && p.slots.empty()) {
    std::vector<ProfSlot> fresh(32768, ProfSlot{nullptr, nullptr, 0});
    bool ok = true;
    for (auto& sl : fresh)
      if (hipEventCreate(&sl.a) != hipSuccess || hipEventCreate(&sl.b) != hipSuccess) { ok = false; break; }
    if (!ok) {                      // nothing half-built is kept: the next enable starts over
      for (auto& sl : fresh) { if (sl.a) (void)hipEventDestroy(sl.a); if (sl.b) (void)hipEventDestroy(sl.b); }
      (void)hipGetLastError();
      p.on = false;
      return ERNIE_EHIP;
    }
    p.slots.swap(fresh);
  }
  p.on = enable != 0;
  p.used = 0;
  for (int c = 0; c < ERNIE_PROF_NCAT; ++c) p.bytes[c] = p.flops[c] = 0.0;
  return ERNIE_OK;
}

int ernie_profile_read(ErnieHandle* h, int category, double* total_ms, int64_t* launches, double* alg_bytes,
                       double* alg_flops) {
  if (!h || category < 0 || category >= ERNIE_PROF_NCAT || !total_ms || !launches) return ERNIE_EINVAL;
  Profiler& p = h->prof;
  double ms = 0.0; int64_t n = 0;
  for (size_t i = 0; i < p.used; ++i) {
    if (p.slots[i].cat != category) continue;
    float t = 0.f;
    if (hipEventSynchronize(p.slots[i].b) != hipSuccess ||
        hipEventElapsedTime(&t, p.slots[i].a, p.slots[i].b) != hipSuccess) return ERNIE_EHIP;
    ms += t; ++n;
  }
  *total_ms = ms; *launches = n;
  if (alg_bytes) *alg_bytes = p.bytes[category];
  if (alg_flops) *alg_flops = p.flops[category];
  return ERNIE_OK;
}

int ernie_debug_handover(int mode, int n_workgroups, int stages, int pieces, int out_units, void* ws_dev, size_t ws_bytes,
                         void* stream, double* us_per_stage, int64_t* bad_units) {
  if ((mode != 0 && mode != 1) || n_workgroups < 8 || n_workgroups > 1024 || stages < 2 || stages > 100000 || out_units < 1 ||
      !ws_dev || !us_per_stage || !bad_units)
    return ERNIE_EINVAL;
  if (pieces != 1 && pieces != 3 && pieces != 6 && pieces != 12) return ERNIE_EINVAL;
  const size_t units = (size_t)n_workgroups * out_units;
  if (units % 64 != 0 || units * 16 * 3 > ((size_t)1 << 31)) return ERNIE_EINVAL;
  const size_t need = units * 16 * 3 + 4096 + 256;
  if (ws_bytes < need || (uintptr_t)ws_dev % 256 != 0) return ERNIE_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(ws_dev);
  unsigned* bufs = reinterpret_cast<unsigned*>(ws);
  unsigned* flags = reinterpret_cast<unsigned*>(ws + units * 16 * 3);
  int* gave_up = reinterpret_cast<int*>(ws + units * 16 * 3 + 4096);
  unsigned* bad = reinterpret_cast<unsigned*>(ws + units * 16 * 3 + 4096 + 64);
  HIP_OK(hipMemsetAsync(ws, 0, need, s));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    if (e0) (void)hipEventDestroy(e0);
    return ERNIE_EHIP;
  }
  float best = 1e30f;
  unsigned epoch0 = 1;
  bool ok = true;
  for (int rep = 0; rep < 4 && ok; ++rep) {
    ok &= hipEventRecord(e0, s) == hipSuccess;
#define PROBE(M, P) hipLaunchKernelGGL((handover_probe_kernel<M, P>), dim3(n_workgroups), dim3(kProbeThreads), 0, s, bufs, \
                                       (unsigned)units, flags, stages, out_units, epoch0, 1u << 18, gave_up, bad)
#define PROBE_BY_P(M) do { if (pieces == 1) PROBE(M, 1); else if (pieces == 3) PROBE(M, 3); else if (pieces == 6) PROBE(M, 6); else PROBE(M, 12); } while (0)
    if (mode == 0) PROBE_BY_P(0); else PROBE_BY_P(1);
#undef PROBE_BY_P
#undef PROBE
    ok &= hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    float ms = 0.f;
    ok &= hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    if (ms < best) best = ms;
    epoch0 += (unsigned)stages + 5;
  }
  int gave = 0; unsigned nbad = 0;
  ok &= hipMemcpyAsync(&gave, gave_up, 4, hipMemcpyDeviceToHost, s) == hipSuccess;
  ok &= hipMemcpyAsync(&nbad, bad, 4, hipMemcpyDeviceToHost, s) == hipSuccess;
  ok &= hipStreamSynchronize(s) == hipSuccess;
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (!ok || launch_status() != ERNIE_OK || gave) return ERNIE_EHIP;
  *us_per_stage = (double)best * 1000.0 / stages;
  *bad_units = nbad;
  return ERNIE_OK;
}

int ernie_debug_tune(ErnieHandle* h, const char* key, int value) {
  if (!h || !key) return ERNIE_EINVAL;
  if (!strcmp(key, "fused_decode")) { h->fused_decode = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "persist")) { h->persist = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "persist_helpers")) { h->persist_helpers = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "persist_dbg")) { h->persist_dbg = value; return ERNIE_OK; }
  if (!strcmp(key, "persist_trace")) { h->persist_trace = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "persist_spin")) { if (value < 1) return ERNIE_EINVAL; h->persist_spin = (unsigned)value; return ERNIE_OK; }
  if (!strcmp(key, "persist_stall")) { if (value < 0 || value > 5) return ERNIE_EINVAL; h->persist_stall = value; return ERNIE_OK; }
  if (!strcmp(key, "dec_nw16")) { h->dec_nw16 = value; return ERNIE_OK; }
  if (!strcmp(key, "big_ln_rows")) { if (value != 1 && value != 2 && value != 4) return ERNIE_EINVAL; h->big_ln_rows = value; return ERNIE_OK; }
  if (!strcmp(key, "big_mfast")) { h->big_mfast = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "big_narrow")) { h->big_narrow = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "big_f1_tile")) { if (value < 0 || value > 2) return ERNIE_EINVAL; h->big_f1_tile = value; return ERNIE_OK; }
  if (!strcmp(key, "pf_tile")) { if (value < 0 || value > 3) return ERNIE_EINVAL; h->pf_tile = value; return ERNIE_OK; }
  if (!strcmp(key, "big_warm")) { if (value < 0 || value > 256) return ERNIE_EINVAL; h->big_warm = value; return ERNIE_OK; }
  if (!strcmp(key, "kv_prefetch")) { if (value < 0 || value > 2048) return ERNIE_EINVAL; h->kv_prefetch = value; return ERNIE_OK; }
  if (!strcmp(key, "dec_prefetch")) { if (value < 0 || value > 1024) return ERNIE_EINVAL; h->dec_prefetch = value; return ERNIE_OK; }
  if (!strcmp(key, "big_logits_gemm")) { h->big_logits_gemm = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "big_f1_fused")) { h->big_f1_fused = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "ln_rpw")) {
    if (value != 0 && value != 1 && value != 2) return ERNIE_EINVAL;
    h->ln_rpw = value;
    return ERNIE_OK;
  }
  if (!strcmp(key, "ln_ns")) {
    if (value != 0 && value != 1 && value != 2 && value != 4) return ERNIE_EINVAL;
    h->ln_ns = value;
    return ERNIE_OK;
  }
  if (!strcmp(key, "attn_nt")) { h->attn_nt = value != 0; return ERNIE_OK; }
  if (!strcmp(key, "attn_dec")) {
    if (value < 0 || value > 5) return ERNIE_EINVAL;
    h->attn_dec = value;
    return ERNIE_OK;
  }
  if (!strcmp(key, "sk_out") || !strcmp(key, "sk_f2")) {
    const int k_tiles = (!strcmp(key, "sk_out") ? h->cfg.d_model : h->cfg.d_ffn) / 16;
    if ((value != 1 && value != 2 && value != 4) || k_tiles % value != 0) return ERNIE_EINVAL;
    (!strcmp(key, "sk_out") ? h->sk_out : h->sk_f2) = value;
    return ERNIE_OK;
  }
  return ERNIE_EINVAL;
}

}  // extern "C"
