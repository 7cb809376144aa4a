// One-launch decode step for small batches (B <= 64): every layer of the step runs inside ONE persistent
// kernel (one workgroup per compute unit), so that the sixty dependent phases of a step are separated by a
// device-memory hand-over (about a microsecond and a half) instead of a kernel boundary (five to seven).
//
// Hand-over protocol.  Every activation matrix that crosses workgroups (the pre-LayerNorm sums, q / k / v,
// the attention output, the GELU output, the residual rows) lives in an exchange buffer of 8-byte pairs
//     { two fp16 values, 32-bit tag }
// where the tag is the number of the decode step (a device-side counter that a later kernel of the same
// stream advances).  A producer writes its pairs with agent-scope stores (they go through to memory instead
// of staying in the XCD's L2); a consumer reads with agent-scope loads (they do not hit stale lines of its
// own XCD's L2) and repeats the load until every tag it got equals this step's tag.  Data and its "ready"
// flag therefore travel in one aligned 8-byte store: no fence, no separate flag, no cache write-back or
// invalidate -- a fence-and-flag hand-over measured 5-6 us on this part, this one 1.4-2.5 us.  Every buffer is
// written exactly once per step (each layer has its own set), so a stale pair always carries an older tag.
// Waits are bounded: after `spin_limit` unsuccessful polls a workgroup writes an error word and leaves, and
// so, in turn, does everyone who waits for it.
//
// Work split.  All five GEMM-shaped phases of a layer use the same decomposition: a workgroup owns R batch
// rows of NS adjacent 32-column strips over the WHOLE contraction (no partial sums cross workgroups); its
// eight waves split the contraction and are added through LDS in a fixed order.  The weight fragments of a
// phase are requested before the workgroup starts polling for the phase's input, so the HBM stream runs under
// the hand-over latency (measured: with the weight loads removed altogether the step is only 13 % shorter;
// warming the L2 for later phases with strided touch loads made it LONGER, because loads return in order and
// every later load of the wave queues behind the touches).  Row-wise work sits where the full row is: LayerNorm in the prologue of the
// consuming GEMM (QKV, FFN1), bias / residual / GELU in the epilogue of the producing one.
#pragma once

#include "attention.h"
#include "common.h"
#include "decode_fused.h"

namespace ernie {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int kAgentScope = 16;        // cache-policy operand of the raw buffer builtins on gfx94x/gfx950: sc1
constexpr int kPersistWaves = 8;
constexpr int kPersistThreads = kPersistWaves * 64;

struct PersistLayer {                   // one per layer, in device memory
  const half_t *wqkv, *wo, *w1, *w2;    // fragment-major
  const float *bqkv, *bo, *b1, *b2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
  half_t *kc, *vc;                      // this layer's key / value cache
};

// A pointer read from device memory (or from a struct passed by value) carries no address space, and loads
// through it are flat instructions (which also count against the LDS counter).  These say "global memory".
template <class T>
__device__ __forceinline__ T* as_global(T* p) {
  typedef __attribute__((address_space(1))) T gT;
  return (T*)(gT*)p;
}
template <class T>
__device__ __forceinline__ T ld_global(const T* p) {
  typedef __attribute__((address_space(1))) const T gT;
  return *(gT*)p;
}
template <class T>
__device__ __forceinline__ void st_global(T* p, T v) {
  typedef __attribute__((address_space(1))) T gT;
  *(gT*)p = v;
}
template <class T>
__device__ __forceinline__ T ld_global_nt(const T* p) {
  typedef __attribute__((address_space(1))) const T gT;
  return __builtin_nontemporal_load((gT*)p);
}
template <bool NT>
__device__ __forceinline__ half8 ld_kv(const half_t* p) {
  if constexpr (NT) return ld_global_nt(reinterpret_cast<const half8*>(p));
  else return ld_global(reinterpret_cast<const half8*>(p));
}

// The thread's index, opaque to the optimiser.  Everything in a phase that derives from the thread or workgroup
// index (offsets, unit numbers) is the same in every layer; hoisted out of the layer loop it would occupy
// registers for the whole kernel, and the spills that follow are reloaded through the same in-order counter
// as the hand-over loads (a reload then waits for every outstanding touch).  Recomputing costs a few ALU
// instructions per phase.
__device__ __forceinline__ int fresh_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}
__device__ __forceinline__ int fresh_wg() {
  int b = blockIdx.x;
  asm volatile("" : "+s"(b));
  return b;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains the vector-memory counter, i.e.
// waits for every outstanding global load and store of the wave: the L2 touches (HBM latency) and the pairs
// just published among them.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Barrier + "did any thread of the workgroup give up a wait?" (sticky: once set, the workgroup leaves).
__device__ __forceinline__ bool persist_sync_fail(bool fail, int* s_fail) {
  if (__any(fail) && (fresh_tid() & 63) == 0) *s_fail = 1;
  lds_barrier();
  return *s_fail != 0;
}

// Per-layer exchange region: [B][cols] fp16 matrices stored as pairs (4 bytes per element), in this order.
struct PersistXch {
  unsigned qkv, o, y1, g, y2, x, x1;    // byte offsets inside a layer's region
  unsigned layer_bytes;
};

struct PersistArgs {
  const PersistLayer* layers;
  int n_layers, B, d, f, H, S;
  float eps;
  // embedding of the fed tokens
  const int* tok; const int* cache_len;
  const half_t* tok_emb; const half_t* pos_emb; const half_t* seg_row;
  const float* emb_g; const float* emb_b;
  int max_pos, vocab_kept, eos;
  int* finished;                        // [B] sticky end-of-sequence flags (may be null when eos < 0)
  const int* slot;                      // cache row of batch row b, or null
  unsigned char* xch; PersistXch xo;
  const unsigned* epoch;                // step counter; this step's tag is *epoch + 1
  half_t* X; float* hidden_out;         // final LayerNorm output [B, d] (plain fp16) and optional fp32 copy
  int* err;                             // host-visible error word (give-up of a bounded wait)
  unsigned spin_limit;
  int stall;                            // test hook: phase number (1..5, layer 0) whose output is withheld; 0 = none
  int attn_nt;
  int dbg;                              // measurement hook, bit mask: 1 = helper workgroups idle, 2 = no weight loads (results are wrong)
  int helpers_from;                     // workgroups from this id on (a multiple of 8) own no unit and warm the L2; = grid if none
  int kv_rows;                          // upper bound of the cache rows of any stream after this step (L2 warm-up only)
  unsigned red_off;                     // byte offset of the cross-wave reduction buffer in dynamic LDS (behind the largest A tile)
  const half_t* table_p; int table_strips;   // packed projection table (32-column strips of K = d) that the next kernel streams, or null
  unsigned long long* trace;            // test hook: [workgroup][layer][32] 100 MHz time stamps (entry, input ready, done per phase), or null
};

// Time stamp `slot` of the workgroup's current layer (tracing only).
__device__ __forceinline__ void persist_stamp(unsigned long long* row, int slot) {
  if (row && threadIdx.x == 0) row[slot] = wall_clock64();
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t xch_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 xch_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kAgentScope);
}
__device__ __forceinline__ void xch_store16(__amdgpu_buffer_rsrc_t r, unsigned byte_off, unsigned p0, unsigned p1, unsigned tag) {
  const u32x4 v = {p0, tag, p1, tag};
  __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, kAgentScope);
}
__device__ __forceinline__ void xch_store8(__amdgpu_buffer_rsrc_t r, unsigned byte_off, unsigned p0, unsigned tag) {
  const u32x2 v = {p0, tag};
  __builtin_amdgcn_raw_buffer_store_b64(v, r, byte_off, 0, kAgentScope);
}
__device__ __forceinline__ bool xch_ready(const u32x4& v, unsigned tag) { return v[1] == tag && v[3] == tag; }
__device__ __forceinline__ unsigned pack_h2(float a, float b) {
  const half2_t h = {(half_t)a, (half_t)b};
  return __builtin_bit_cast(unsigned, h);
}
__device__ __forceinline__ void unpack_h2(unsigned w, float& a, float& b) {
  const half2_t h = __builtin_bit_cast(half2_t, w);
  a = (float)h[0]; b = (float)h[1];
}

// Cross-lane moves on the vector ALU's data-parallel path (a few cycles each; the LDS crossbar behind __shfl_xor
// costs a hundred and its own wait).  Lane layouts checked on the device with an in-bounds probe.
template <int CTRL>
__device__ __forceinline__ float lane_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_xor1(float v) { return lane_dpp<0xB1>(v); }     // quad_perm [1, 0, 3, 2]
__device__ __forceinline__ float lane_xor8(float v) { return lane_dpp<0x128>(v); }    // row_ror 8: lane ^ 8 inside a row of 16
// Sum over each aligned group of eight lanes, in every lane of the group.
__device__ __forceinline__ float team8_sum(float v) {
  v += lane_dpp<0xB1>(v);       // lane ^ 1
  v += lane_dpp<0x4E>(v);       // lane ^ 2 (quad_perm [2, 3, 0, 1])
  v += lane_dpp<0x141>(v);      // row_half_mirror: the other quad of the eight
  return v;
}
struct LanePair { float a, b; };
// Rows of 16 lanes r0..r3 of v: a = {r0, r0, r2, r2}, b = {r1, r1, r3, r3} (every lane sees its own row and the row ^ 1).
__device__ __forceinline__ LanePair rows_swap16(float v) {
  const unsigned x = __builtin_bit_cast(unsigned, v);
  const u32x2 r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  const unsigned a = r[0], b = r[1];      // (a bit cast applied to a vector element directly reads element 0)
  return {__builtin_bit_cast(float, a), __builtin_bit_cast(float, b)};
}
// Halves of 32 lanes: a = {low, low}, b = {high, high}.
__device__ __forceinline__ LanePair halves_swap32(float v) {
  const unsigned x = __builtin_bit_cast(unsigned, v);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  const unsigned a = r[0], b = r[1];
  return {__builtin_bit_cast(float, a), __builtin_bit_cast(float, b)};
}
// Sum over the 64 lanes, the same bits in every lane.
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v = team8_sum(v);
  v += lane_dpp<0x140>(v);      // row_mirror: the other eight of the row
  const LanePair r = rows_swap16(v);
  v = r.a + r.b;
  const LanePair h = halves_swap32(v);
  return h.a + h.b;
}

enum { PRO_LN = 0, PRO_EMBED = 1, PRO_COPY = 2 };
enum { PEPI_BIAS = 0, PEPI_RES = 1, PEPI_GELU = 2 };

struct PersistGemm {
  const half_t* Wp; int N, K, B;
  const unsigned char* in; const float* gamma; const float* beta; float eps;     // prologue
  unsigned char* xout;                 // PRO_LN / PRO_EMBED: normalised rows as pairs (each strip group writes its share of the columns)
  const float* bias;                   // [N]
  const unsigned char* res;            // PEPI_RES: residual rows [B][N] as pairs
  unsigned char* out;                  // [B][N] as pairs
  bool withhold;                       // test hook: compute, but do not publish
};

// The weight fragments a wave holds for its unit of a GEMM phase: NS strips x FR k-tiles, requested one
// phase ahead (right after the current phase's input has arrived), so that they have landed by the time the
// next phase's input does.  Loads return in order: a poll issued behind a late weight request would wait for it.
template <int NS, int FR>
struct PersistW {
  half8 w[NS][FR];
};

// A workgroup's unit of a GEMM phase.  Every phase has at most as many units as unit-owning workgroups (the host checks), so a
// workgroup owns one unit or sits the phase out.  Units are (strip group, row group) in XCD-contiguous order
// with the row group fastest: the row groups of a strip group run on one XCD and share its weight fragments
// in that L2.
template <int R, int NS>
struct PersistUnit {
  static constexpr int NV = R <= 8 ? 4 : R / 2;      // accumulator registers that hold rows < R (row = 8 (v / 4) + 4 (lane / 32) + v % 4)
  static constexpr int kMyNv = (NS * NV + kPersistWaves - 1) / kPersistWaves;
  int sg, row0;
  bool has;
  float bias_r[kMyNv];        // bias of this lane's output columns, fetched ahead of the epilogue
};

template <int R, int NS>
__device__ __forceinline__ PersistUnit<R, NS> persist_unit(int N, int B, const float* bias) {
  PersistUnit<R, NS> u;
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_tiles = N / 32, zg = (B + R - 1) / R, n_units = ((n_tiles + NS - 1) / NS) * zg;
  const int wg = fresh_wg();
  u.has = wg < n_units;
  const int logical = u.has ? xcd_contiguous_id(wg, n_units) : 0;      // (n_units <= the unit-owning workgroups, host-checked)
  u.sg = logical / zg;
  u.row0 = (logical - u.sg * zg) * R;
#pragma unroll
  for (int i = 0; i < PersistUnit<R, NS>::kMyNv; ++i) {
    const int nt = u.sg * NS + (wave + i * kPersistWaves) / PersistUnit<R, NS>::NV;
    u.bias_r[i] = ld_global(bias + min(nt * 32 + (lane & 31), N - 1));
  }
  return u;
}

// Requests the workgroup's weight fragments of a phase (all of them when the wave's share of the contraction
// is at most FR k-tiles, which the host guarantees).  Straight-line: a workgroup that sits the phase out loads
// its clamped unit's fragments too (a few KB from L2) rather than branching, so that the registers have one
// definition.
template <int R, int NS, int FR>
__device__ __forceinline__ void persist_w_issue(PersistW<NS, FR>& W, const half_t* Wp, int N, int K, int B, bool off = false) {
  if (off) {
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int n = 0; n < NS; ++n)
#pragma unroll
      for (int u = 0; u < FR; ++u) W.w[n][u] = z;
    return;
  }
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k_tiles = K / 16, n_tiles = N / 32;
  const int zg = (B + R - 1) / R, n_units = ((n_tiles + NS - 1) / NS) * zg;
  const int wg = fresh_wg();
  const int logical = wg < n_units ? xcd_contiguous_id(wg, n_units) : 0;
  const int sg = logical / zg;
  const int kb = k_tiles * wave / kPersistWaves;
#pragma unroll
  for (int n = 0; n < NS; ++n) {
    const half_t* wp = Wp + packed_frag_offset(min(sg * NS + n, n_tiles - 1), 0, k_tiles) + lane * 8;
#pragma unroll
    for (int u = 0; u < FR; ++u) W.w[n][u] = ld_global(reinterpret_cast<const half8*>(wp + (size_t)min(kb + u, k_tiles - 1) * 512));
  }
}

// First half of a GEMM phase: waits for the unit's input and leaves the A tile [R][K] as fp16 in LDS (PRO_LN /
// PRO_EMBED: normalised, and published as residual rows, a share of the columns per strip group; PRO_COPY: copied, plus the
// residual tile of the epilogue).  Returns false (uniformly for the workgroup) when a wait gave up.
template <int R, int NS, int PRO, int EPI, int PC = 4, int RC = 2>
__device__ __forceinline__ bool persist_gemm_in(const PersistGemm& g, const PersistArgs& p, unsigned tag,
                                                unsigned char* smem_raw, half_t* sRes, int* s_fail,
                                                const PersistUnit<R, NS>& un) {
  constexpr int NW = kPersistWaves;
  constexpr int RPW = R / NW;                 // LayerNorm prologues: rows per wave
  static_assert(PRO == PRO_COPY || R == 8 || R == 16, "LayerNorm prologue: one or two rows per wave");
  static_assert(EPI != PEPI_RES || NS == 1, "the residual tile is one strip wide");
  half_t* sA = reinterpret_cast<half_t*>(smem_raw);            // [R][K + 8]
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = g.K, B = g.B, N = g.N, pitch = K + 8;
  const int sg = un.sg, row0 = un.row0;
  const __amdgpu_buffer_rsrc_t r_in = xch_rsrc(g.in, (unsigned)B * K * 4);
  const __amdgpu_buffer_rsrc_t r_xout = xch_rsrc(g.xout, (unsigned)B * K * 4);
  const __amdgpu_buffer_rsrc_t r_res = xch_rsrc(g.res, (unsigned)B * N * 4);
  bool fail = false;
  if (un.has) {
    if constexpr (PRO == PRO_COPY) {
      const int upr = K / 4;                         // 16-byte units (4 values) per row
      const int total = R * upr;
      constexpr int kPieces = PC > 8 ? (PC + 1) / 2 : PC;      // PC = 16-byte units per thread of the whole tile: one poll round
      const int n_res = EPI == PEPI_RES ? R * 8 : 0; // residual tile: R rows x 32 columns = R * 8 units
      u32x4 rv = {0, 0, 0, 0};
      const int rr_res = min(row0 + tid / 8, B - 1);
      const unsigned res_off = ((unsigned)rr_res * N + sg * 32 + (tid & 7) * 4) * 4;
      bool res_pending = tid < n_res;
      for (int base = 0; base < total; base += kPersistThreads * kPieces) {      // uniform trip count
        const int id0 = base + tid;
        u32x4 v[kPieces];
        unsigned off[kPieces];
        int dst[kPieces];
#pragma unroll
        for (int q = 0; q < kPieces; ++q) {
          const int id = (int)((unsigned)(id0 + q * kPersistThreads) % (unsigned)total);         // past the tile: a duplicate is loaded, not stored
          const int r = id / upr, c4 = id - r * upr;
          off[q] = ((unsigned)min(row0 + r, B - 1) * K + c4 * 4) * 4;
          dst[q] = r * pitch + c4 * 4;
        }
        // (Reading only the pieces that were missing in the round before, or waiting on one piece before fetching
        // the rest, both measured slower than repeating the whole round.)
        unsigned spins = 0;
        while (true) {
          asm volatile("" ::: "memory");
#pragma unroll
          for (int q = 0; q < kPieces; ++q) v[q] = xch_load16(r_in, off[q]);
          if (res_pending) rv = xch_load16(r_res, res_off);
          bool ok = !res_pending || xch_ready(rv, tag);
#pragma unroll
          for (int q = 0; q < kPieces; ++q) ok &= xch_ready(v[q], tag);
          if (__all(ok)) break;
          if (++spins > p.spin_limit) { fail = true; break; }
        }
        if (fail) break;
#pragma unroll
        for (int q = 0; q < kPieces; ++q)
          if (id0 + q * kPersistThreads < total) {
            const u32x2 w = {v[q][0], v[q][2]};
            *reinterpret_cast<u32x2*>(sA + dst[q]) = w;
          }
        if (res_pending) {
          const u32x2 w = {rv[0], rv[2]};
          *reinterpret_cast<u32x2*>(sRes + (tid / 8) * 32 + (tid & 7) * 4) = w;
          res_pending = false;
        }
      }
    } else {
      // wave w normalises rows row0 + w * RPW + i; chunk c of lane l covers features (c * 64 + l) * 8 .. + 7
      const int chunks = K / 8;
      float v[RPW][RC][8], gm[RC][8], bt[RC][8];
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        const int cc = min(c * 64 + lane, chunks - 1);
        const floatx4 g0 = ld_global(reinterpret_cast<const floatx4*>(g.gamma + cc * 8)), g1 = ld_global(reinterpret_cast<const floatx4*>(g.gamma + cc * 8 + 4));
        const floatx4 t0 = ld_global(reinterpret_cast<const floatx4*>(g.beta + cc * 8)), t1 = ld_global(reinterpret_cast<const floatx4*>(g.beta + cc * 8 + 4));
#pragma unroll
        for (int j = 0; j < 4; ++j) { gm[c][j] = g0[j]; gm[c][4 + j] = g1[j]; bt[c][j] = t0[j]; bt[c][4 + j] = t1[j]; }
      }
      if constexpr (PRO == PRO_EMBED) {
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
          const int r = row0 + wave * RPW + i, rr = min(r, B - 1);
          const int id = min(max(p.tok[rr], 0), p.vocab_kept - 1);
          const int pos = min(p.cache_len[rr], p.max_pos - 1);
          if (p.eos >= 0 && sg == 0 && lane == 0 && r < B && p.tok[rr] == p.eos) p.finished[rr] = 1;
#pragma unroll
          for (int c = 0; c < RC; ++c) {
            const int cc = min(c * 64 + lane, chunks - 1);
            const half8 e = ld_global(reinterpret_cast<const half8*>(p.tok_emb + (size_t)id * K + cc * 8));
            const half8 q = ld_global(reinterpret_cast<const half8*>(p.pos_emb + (size_t)pos * K + cc * 8));
            half8 s8 = {0, 0, 0, 0, 0, 0, 0, 0};
            if (p.seg_row) s8 = ld_global(reinterpret_cast<const half8*>(p.seg_row + cc * 8));
            const float live = (c * 64 + lane < chunks) ? 1.f : 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[i][c][j] = ((float)e[j] + (float)q[j] + (float)s8[j]) * live;
          }
        }
      } else {
        u32x4 a[RPW][RC][2] = {};
        unsigned off[RPW][RC];
#pragma unroll
        for (int i = 0; i < RPW; ++i)
#pragma unroll
          for (int c = 0; c < RC; ++c)
            off[i][c] = ((unsigned)min(row0 + wave * RPW + i, B - 1) * K + min(c * 64 + lane, chunks - 1) * 8) * 4;
        unsigned spins = 0;
        while (true) {
          asm volatile("" ::: "memory");
          bool ok = true;
#pragma unroll
          for (int i = 0; i < RPW; ++i)
#pragma unroll
            for (int c = 0; c < RC; ++c) {
              a[i][c][0] = xch_load16(r_in, off[i][c]);
              a[i][c][1] = xch_load16(r_in, off[i][c] + 16);
            }
#pragma unroll
          for (int i = 0; i < RPW; ++i)
#pragma unroll
            for (int c = 0; c < RC; ++c) ok &= xch_ready(a[i][c][0], tag) && xch_ready(a[i][c][1], tag);
          if (__all(ok)) break;
          if (++spins > p.spin_limit) { fail = true; break; }
        }
#pragma unroll
        for (int i = 0; i < RPW; ++i)
#pragma unroll
          for (int c = 0; c < RC; ++c) {
            const float live = (c * 64 + lane < chunks) ? 1.f : 0.f;     // the duplicated tail chunk stays out of the sums
            unpack_h2(a[i][c][0][0], v[i][c][0], v[i][c][1]); unpack_h2(a[i][c][0][2], v[i][c][2], v[i][c][3]);
            unpack_h2(a[i][c][1][0], v[i][c][4], v[i][c][5]); unpack_h2(a[i][c][1][2], v[i][c][6], v[i][c][7]);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[i][c][j] *= live;
          }
      }
      float mean[RPW], rstd[RPW];
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < RC; ++c)
#pragma unroll
          for (int j = 0; j < 8; ++j) sum += v[i][c][j];
        mean[i] = sum;
      }
#pragma unroll
      for (int i = 0; i < RPW; ++i) mean[i] = wave_sum_dpp(mean[i]);
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        mean[i] /= (float)K;
        float q = 0.f;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
          const float live = (c * 64 + lane < chunks) ? 1.f : 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) { const float t = (v[i][c][j] - mean[i]) * live; q += t * t; }
        }
        rstd[i] = q;
      }
#pragma unroll
      for (int i = 0; i < RPW; ++i) rstd[i] = wave_sum_dpp(rstd[i]);
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        const int r = row0 + wave * RPW + i;
        const float rs = rsqrtf(rstd[i] / (float)K + g.eps);
        // every strip group of the row group holds the whole normalised row: each publishes its share of the
        // residual copy (one group writing all of it ran a microsecond behind the others in every phase)
        const int n_sg = (N / 32 + NS - 1) / NS;
        const int ch_lo = sg * chunks / n_sg, ch_hi = (sg + 1) * chunks / n_sg;
        const bool writer = r < B && !fail;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
          const int ch = c * 64 + lane;
          if (ch < chunks) {
            half8 o;
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = (half_t)((v[i][c][j] - mean[i]) * rs * gm[c][j] + bt[c][j]);
            *reinterpret_cast<half8*>(sA + (wave * RPW + i) * pitch + ch * 8) = o;
            if (writer && ch >= ch_lo && ch < ch_hi) {
              const u32x4 w = __builtin_bit_cast(u32x4, o);
              const unsigned off = ((unsigned)r * K + ch * 8) * 4;
              xch_store16(r_xout, off, w[0], w[1], tag);
              xch_store16(r_xout, off + 16, w[2], w[3], tag);
            }
          }
        }
      }
    }
  }
  return !persist_sync_fail(fail, s_fail);
}

// Second half of a GEMM phase: MFMA over each wave's share of the contraction, cross-wave reduction through
// LDS in a fixed order, bias / residual / GELU, and publication of the unit's outputs as tagged pairs.
// The MFMA loop is branch-free: FR k-steps are always issued, a step past the wave's share with a zero A
// fragment, so that all LDS fragment reads are in flight before the first product and nothing but the
// matrix pipe paces the loop.  With one strip per workgroup the steps alternate between two accumulators
// (a chain of dependent MFMAs issues one per result latency, not one per pass through the pipe).
template <int R, int NS, int FR, int EPI>
__device__ __forceinline__ void persist_gemm_out(const PersistGemm& g, unsigned tag, unsigned char* smem_raw, float* red,
                                                 const half_t* sRes, const PersistUnit<R, NS>& un, PersistW<NS, FR>& W,
                                                 unsigned long long* tr = nullptr, int slot0 = 0) {
  constexpr int NW = kPersistWaves;
  constexpr int NV = PersistUnit<R, NS>::NV, kMyNv = PersistUnit<R, NS>::kMyNv;
  constexpr int NA = NS == 1 ? 2 : NS;        // independent accumulator chains
  const half_t* sA = reinterpret_cast<const half_t*>(smem_raw);
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = g.K, B = g.B, N = g.N;
  const int k_tiles = K / 16, n_tiles = N / 32, pitch = K + 8;
  const int kb = k_tiles * wave / NW, ke = k_tiles * (wave + 1) / NW;      // ke - kb <= FR (host-checked)
  const __amdgpu_buffer_rsrc_t r_out = xch_rsrc(g.out, (unsigned)B * N * 4);
  if (un.has) {
    floatx16 acc[NA];
#pragma unroll
    for (int n = 0; n < NA; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    const half_t* ap = sA + (lane & (R - 1)) * pitch + 8 * (lane >> 5);    // tile rows R..31 repeat rows 0..R-1
    // A fragments are read eight k-steps ahead of their products (all of them would cost four registers per step)
    constexpr int kAhead = FR < 8 ? FR : 8;
    half8 af[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) af[u] = *reinterpret_cast<const half8*>(ap + min(kb + u, k_tiles - 1) * 16);
#pragma unroll
    for (int u = 0; u < FR; ++u) {
      const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      const half8 a = (kb + u < ke) ? af[u % kAhead] : z;
      if (u + kAhead < FR) af[u % kAhead] = *reinterpret_cast<const half8*>(ap + min(kb + u + kAhead, k_tiles - 1) * 16);
      if constexpr (NS == 1) acc[u & 1] = mfma32(a, W.w[0][u], acc[u & 1]);
      else {
#pragma unroll
        for (int n = 0; n < NS; ++n) acc[n] = mfma32(a, W.w[n][u], acc[n]);
      }
    }
    if constexpr (NS == 1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[0][v] += acc[1][v];
    }
    persist_stamp(tr, slot0);
    // `red` does not overlap the A tile: no barrier between the last fragment read and the first partial
#pragma unroll
    for (int n = 0; n < NS; ++n)
#pragma unroll
      for (int v = 0; v < NV; ++v) red[(wave * NS * NV + n * NV + v) * 64 + lane] = acc[n][v];
    lds_barrier();
    persist_stamp(tr, slot0 + 2);
#pragma unroll
    for (int i = 0; i < kMyNv; ++i) {
      const int nv = wave + i * NW;
      if (nv >= NS * NV) break;
      const int n = nv / NV, v = nv - n * NV;
      const int nt = un.sg * NS + n;
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += red[(w * NS * NV + nv) * 64 + lane];
      const int tr_ = mfma32_row(v, lane);                // row inside the tile
      const int row = un.row0 + tr_, col = nt * 32 + (lane & 31);
      const bool live = nt < n_tiles && tr_ < R && row < B;
      float val = s + un.bias_r[i];
      if constexpr (EPI == PEPI_RES) val += (float)sRes[min(tr_, R - 1) * 32 + (lane & 31)];
      if constexpr (EPI == PEPI_GELU) val = gelu_erf_fast(val);
      const float nb = lane_xor1(val);                    // the odd neighbour column
      if (live && (lane & 1) == 0 && !g.withhold)
        xch_store8(r_out, ((unsigned)row * N + col) * 4, pack_h2(val, nb), tag);
    }
    persist_stamp(tr, slot0 + 3);
  }
  lds_barrier();          // the A tile, `red` and the residual tile are free for the next phase
}

// The first batch of cache rows of a workgroup's first pair of streams, and the streams' cached length,
// requested a phase ahead like the weight fragments.
template <int U>
struct PersistKV {
  half8 k[U], v[U];
  int len;
};

template <int U, bool NT>
__device__ __forceinline__ void persist_kv_issue(PersistKV<U>& F, const PersistArgs& p, const PersistLayer& L, int u0) {
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, w4 = wave & 3, ec = lane & 7, team = lane >> 3;
  const int H = p.H, S = p.S;
  const int s = min(u0 * 2 + grp, p.B * H - 1);        // clamped: a group without a stream loads a valid one and ignores it
  const int b = s / H, h = s - b * H;
  const int cb = p.slot ? p.slot[b] : b;
  const half_t* Kb = L.kc + ((size_t)cb * H + h) * S * 64 + ec * 8;
  const half_t* Vb = L.vc + ((size_t)cb * H + h) * S * 64 + ec * 8;
  // Rows past the cached length are not requested (their lane repeats the last written row and gives it weight
  // zero): what a lane holds is always data some step has written, never arbitrary bits.
  const int len = min(ld_global(p.cache_len + b), S);
  const int last = max(len - 1, 0);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t row = (size_t)min((w4 * U + u) * 8 + team, last) * 64;
    F.k[u] = ld_kv<NT>(Kb + row);
    F.v[u] = ld_kv<NT>(Vb + row);
  }
  F.len = len;
}

__device__ __forceinline__ half2_t half_pair(const half8& v, int j) {
  const half2_t r = {v[2 * j], v[2 * j + 1]};
  return r;
}

// q (scaled), k, v of the new token of one stream, as the attention uses them.
struct PersistQKV {
  half2_t q[4];           // scaled by 1/8 (exact in fp16)
  half8 knew, vnew;
};

// Waits for q, k, v of stream (b, h) in the exchange buffer; false when the wait gave up.
__device__ __forceinline__ bool persist_qkv_wait(PersistQKV& o, const PersistArgs& p, __amdgpu_buffer_rsrc_t r_qkv, int b,
                                                 int h, unsigned tag) {
  const int ec = fresh_tid() & 7, d = p.d;
  const unsigned off = ((unsigned)b * 3 * d + h * 64 + ec * 8) * 4;
  u32x4 a[3][2] = {};
  unsigned spins = 0;
  bool good = true;
  while (true) {
    asm volatile("" ::: "memory");
    bool ok = true;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      a[t][0] = xch_load16(r_qkv, off + (unsigned)t * d * 4);
      a[t][1] = xch_load16(r_qkv, off + (unsigned)t * d * 4 + 16);
    }
#pragma unroll
    for (int t = 0; t < 3; ++t) ok &= xch_ready(a[t][0], tag) && xch_ready(a[t][1], tag);
    if (__all(ok)) break;
    if (++spins > p.spin_limit) { good = false; break; }
  }
  const half2_t eighth = {(half_t)0.125f, (half_t)0.125f};
  const unsigned q01 = a[0][0][0], q23 = a[0][0][2], q45 = a[0][1][0], q67 = a[0][1][2];   // (scalars first: a bit cast applied to a vector element directly reads element 0)
  o.q[0] = __builtin_bit_cast(half2_t, q01) * eighth; o.q[1] = __builtin_bit_cast(half2_t, q23) * eighth;
  o.q[2] = __builtin_bit_cast(half2_t, q45) * eighth; o.q[3] = __builtin_bit_cast(half2_t, q67) * eighth;
  const u32x4 kw = {a[1][0][0], a[1][0][2], a[1][1][0], a[1][1][2]};
  const u32x4 vw = {a[2][0][0], a[2][0][2], a[2][1][0], a[2][1][2]};
  o.knew = __builtin_bit_cast(half8, kw);
  o.vnew = __builtin_bit_cast(half8, vw);
  return good;
}

// One (sequence, head) stream by a group of four waves: online softmax over the cache rows in F (first batch)
// and the batches after it, the new key / value appended and used from registers; the group's wave 0 ends up
// with the merged state after the workgroup barrier, which the caller provides.
template <int U, bool NT>
__device__ __forceinline__ void persist_attn_stream(SoftmaxPart& st, const PersistKV<U>& F, const PersistQKV& x,
                                                    half_t* Kb, half_t* Vb, int S, float (*sm)[8][10]) {
  constexpr int NW = 4;
  const int tid = fresh_tid(), lane = tid & 63;
  const int w4 = __builtin_amdgcn_readfirstlane(tid >> 6) & 3;
  const int ec = lane & 7, team = lane >> 3;
  half8 kf[U], vf[U];
  int key[U];
  int g0 = w4 * U;
#pragma unroll
  for (int u = 0; u < U; ++u) { key[u] = (g0 + u) * 8 + team; kf[u] = F.k[u]; vf[u] = F.v[u]; }
  const int len = F.len;                        // cached rows (at most S)
  const bool has_new = len < S;                 // a replayed step past capacity appends nothing
  const int last = max(len - 1, 0);
  if (len == 0) {                               // nothing cached yet: the repeated "last row" is unwritten memory
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < U; ++u) vf[u] = z;
  }
  if (has_new && w4 == 0 && team == 0) {
    st_global(reinterpret_cast<half8*>(Kb + (size_t)len * 64), x.knew);
    st_global(reinterpret_cast<half8*>(Vb + (size_t)len * 64), x.vnew);
  }
  // the new token's own key and value come from registers: one team of one wave takes them as an extra term
  const bool mine_new = has_new && w4 == 0 && team == 0;
  float sc_new;
  {
    float pr = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) pr = __builtin_amdgcn_fdot2(x.q[j], half_pair(x.knew, j), pr, false);
    pr = team8_sum(pr);
    sc_new = mine_new ? pr : -INFINITY;
  }
  bool first = true;
  // One running maximum for the whole wave (every lane holds the same st.m): the eight teams' partial sums then
  // share a scale and are simply added at the end, instead of merged pairwise with their own maxima.
  while (first || g0 * 8 < len) {
    float sc[U];
    float mx = first ? sc_new : -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float pr = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) pr = __builtin_amdgcn_fdot2(x.q[j], half_pair(kf[u], j), pr, false);
      pr = team8_sum(pr);
      sc[u] = key[u] < len ? pr : -INFINITY;
      mx = fmaxf(mx, sc[u]);
    }
    half8 vcur[U];
#pragma unroll
    for (int u = 0; u < U; ++u) vcur[u] = vf[u];
    g0 += NW * U;
    if (g0 * 8 < len) {                          // next batch in flight during the softmax update
#pragma unroll
      for (int u = 0; u < U; ++u) {
        key[u] = (g0 + u) * 8 + team;
        const size_t row = (size_t)min(key[u], last) * 64;
        kf[u] = ld_kv<NT>(Kb + row);
        vf[u] = ld_kv<NT>(Vb + row);
      }
    }
    {  // maximum over the eight teams (the lanes of a team agree already)
      mx = fmaxf(mx, lane_xor8(mx));
      const LanePair r = rows_swap16(mx);
      mx = fmaxf(r.a, r.b);
      const LanePair hh = halves_swap32(mx);
      mx = fmaxf(st.m, fmaxf(hh.a, hh.b));
    }
    if (mx != -INFINITY) {                       // uniform for the wave
      const float alpha = (st.m == -INFINITY) ? 0.f : __expf(st.m - mx);
      st.l *= alpha;
#pragma unroll
      for (int j = 0; j < 8; ++j) st.acc[j] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float pr = __expf(sc[u] - mx);
        st.l += pr;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[j] += pr * (float)vcur[u][j];
      }
      if (first) {
        const float pr = __expf(sc_new - mx);    // zero except in the one team that owns the new token
        st.l += pr;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[j] += pr * (float)x.vnew[j];
      }
      st.m = mx;
    }
    first = false;
  }
  {  // sums over the eight teams: lane ^ 8, then row ^ 1, then half ^ 1 (each lane keeps its eight features)
    st.l += lane_xor8(st.l);
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j] += lane_xor8(st.acc[j]);
    {
      const LanePair l = rows_swap16(st.l);
      st.l = l.a + l.b;
#pragma unroll
      for (int j = 0; j < 8; ++j) { const LanePair a = rows_swap16(st.acc[j]); st.acc[j] = a.a + a.b; }
    }
    {
      const LanePair l = halves_swap32(st.l);
      st.l = l.a + l.b;
#pragma unroll
      for (int j = 0; j < 8; ++j) { const LanePair a = halves_swap32(st.acc[j]); st.acc[j] = a.a + a.b; }
    }
  }
  if (team == 0) {
    sm[w4][ec][0] = st.m; sm[w4][ec][1] = st.l;
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[w4][ec][2 + j] = st.acc[j];
  }
}

// Publishes one stream's attention output (merged over the group's waves) as tagged pairs; a finished
// sequence's row is zeros (unused, but its consumers still wait for the tag).
__device__ __forceinline__ void persist_attn_publish(SoftmaxPart& st, float (*sm)[8][10], bool done, bool withhold,
                                                     __amdgpu_buffer_rsrc_t r_o, int b, int h, int d, unsigned tag) {
  const int ec = fresh_tid() & 7;
  float o8[8];
  if (done) {
#pragma unroll
    for (int j = 0; j < 8; ++j) o8[j] = 0.f;
  } else {
    // the four waves' partial sums in one level: a common maximum, four independent scales
    const float m1 = sm[1][ec][0], m2 = sm[2][ec][0], m3 = sm[3][ec][0];
    const float mx = fmaxf(fmaxf(st.m, m1), fmaxf(m2, m3));
    const float s0 = __expf(st.m - mx), s1 = __expf(m1 - mx), s2 = __expf(m2 - mx), s3 = __expf(m3 - mx);   // a wave without keys has m = -inf: scale 0
    const float l = st.l * s0 + sm[1][ec][1] * s1 + sm[2][ec][1] * s2 + sm[3][ec][1] * s3;
    const float inv = __builtin_amdgcn_rcpf(l);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      o8[j] = (st.acc[j] * s0 + sm[1][ec][2 + j] * s1 + sm[2][ec][2 + j] * s2 + sm[3][ec][2 + j] * s3) * inv;
  }
  if (!withhold) {
    const unsigned off = ((unsigned)b * d + h * 64 + ec * 8) * 4;
    xch_store16(r_o, off, pack_h2(o8[0], o8[1]), pack_h2(o8[2], o8[3]), tag);
    xch_store16(r_o, off + 16, pack_h2(o8[4], o8[5]), pack_h2(o8[6], o8[7]), tag);
  }
}

// Attention of pair `u0` of streams (two groups of four waves).  With `F_ready` the first batch of cache rows is
// already in F (requested a phase ago); otherwise it is requested here.  `x` holds q, k, v when `x_ready`.
template <int U, bool NT>
__device__ __forceinline__ bool persist_attn_pair(const PersistArgs& p, const PersistLayer& L, unsigned char* xl, unsigned tag,
                                                  bool withhold, int u0, PersistKV<U>& F, bool F_ready, PersistQKV& x,
                                                  bool x_ready, bool x_good, float (*sm_all)[4][8][10], int* s_fail,
                                                  unsigned long long* tr = nullptr) {
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, w4 = wave & 3, ec = lane & 7, team = lane >> 3;
  const int B = p.B, H = p.H, S = p.S, d = p.d, n_streams = B * H;
  const __amdgpu_buffer_rsrc_t r_qkv = xch_rsrc(xl + p.xo.qkv, (unsigned)B * 3 * d * 4);
  const __amdgpu_buffer_rsrc_t r_o = xch_rsrc(xl + p.xo.o, (unsigned)B * d * 4);
  const int s = u0 * 2 + grp;
  const bool active = s < n_streams;
  const int sc = min(s, n_streams - 1), b = sc / H, h = sc - b * H;
  // a sequence that is fed the end token (now or at an earlier step) is finished: no cache stream, no append
  const bool done = active && p.eos >= 0 && (p.finished[b] != 0 || p.tok[b] == p.eos);
  persist_stamp(tr, 28);
  if (!F_ready) persist_kv_issue<U, NT>(F, p, L, u0);
  bool good = x_good;
  if (!x_ready && active && !done) good = persist_qkv_wait(x, p, r_qkv, b, h, tag);
  SoftmaxPart st;
  st.m = -INFINITY; st.l = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] = 0.f;
  if (active && !done && good) {
    const int cb = p.slot ? p.slot[b] : b;
    half_t* Kb = L.kc + ((size_t)cb * H + h) * S * 64 + ec * 8;
    half_t* Vb = L.vc + ((size_t)cb * H + h) * S * 64 + ec * 8;
    persist_attn_stream<U, NT>(st, F, x, Kb, Vb, S, sm_all[grp]);
  }
  persist_stamp(tr, 29);
  if (persist_sync_fail(!good, s_fail)) return false;
  persist_stamp(tr, 30);
  if (active && w4 == 0 && team == 0) persist_attn_publish(st, sm_all[grp], done, withhold, r_o, b, h, d, tag);
  lds_barrier();          // `sm` is free for the next pair of streams
  return true;
}

// Final LayerNorm of the step: one wave per row reads the last layer's pre-LayerNorm sums from the exchange
// buffer and writes the plain fp16 rows the projection kernel reads (and the caller's fp32 copy).
template <int RC>
__device__ __forceinline__ bool persist_final_ln(const PersistArgs& p, const PersistLayer& L, const unsigned char* y2,
                                                 unsigned tag, int* s_fail) {
  const int tid = fresh_tid(), lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = p.d, B = p.B, chunks = d / 8;
  const __amdgpu_buffer_rsrc_t r_in = xch_rsrc(y2, (unsigned)B * d * 4);
  bool fail = false;
  for (int r = blockIdx.x * kPersistWaves + wave; r < B; r += p.helpers_from * kPersistWaves) {
    u32x4 a[RC][2];
    unsigned spins = 0;
    while (true) {
      asm volatile("" ::: "memory");
      bool ok = true;
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        const unsigned off = ((unsigned)r * d + min(c * 64 + lane, chunks - 1) * 8) * 4;
        a[c][0] = xch_load16(r_in, off);
        a[c][1] = xch_load16(r_in, off + 16);
      }
#pragma unroll
      for (int c = 0; c < RC; ++c) ok &= xch_ready(a[c][0], tag) && xch_ready(a[c][1], tag);
      if (__all(ok)) break;
      if (++spins > p.spin_limit) { fail = true; break; }
    }
    if (fail) break;
    RowRegs<RC> v;
#pragma unroll
    for (int c = 0; c < RC; ++c) {
      unpack_h2(a[c][0][0], v.v[c][0], v.v[c][1]); unpack_h2(a[c][0][2], v.v[c][2], v.v[c][3]);
      unpack_h2(a[c][1][0], v.v[c][4], v.v[c][5]); unpack_h2(a[c][1][2], v.v[c][6], v.v[c][7]);
    }
    row_layernorm_store(v, d, lane, L.ln2_g, L.ln2_b, p.eps, p.X + (size_t)r * d);
    if (p.hidden_out) {
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        const int ch = c * 64 + lane;
        if (ch < chunks) {
          const half8 o = *reinterpret_cast<const half8*>(p.X + (size_t)r * d + ch * 8);
#pragma unroll
          for (int j = 0; j < 8; ++j) p.hidden_out[(size_t)r * d + ch * 8 + j] = (float)o[j];
        }
      }
    }
  }
  return !persist_sync_fail(fail, s_fail);
}

// ---------------------------------------------------------------- helper workgroups
// Workgroups past the largest phase never own a unit.  They run ahead of the others and pull what the coming
// phases will read out of HBM into the L2 of the XCD that will read it (workgroup ids congruent mod 8 share an
// XCD, and a unit's workgroup is known in advance): one 4-byte load per 64 bytes, values discarded.  Their own
// loads queue behind their touches, which delays nobody.  The others then request their weight fragments and
// cache rows at the usual place and find them in L2.
//
// Touches up to 16 x 32 KB of [base, base + bytes) (the rest is left to the consumer).
__device__ __forceinline__ void persist_helper_touch(const unsigned char* base, size_t bytes) {
  if (bytes == 0) return;
  const size_t lines = (bytes + 63) / 64;
  const int tid = threadIdx.x;
  constexpr int kFlight = 16;
  for (size_t l0 = 0; l0 < lines; l0 += (size_t)kFlight * kPersistThreads) {
    unsigned t[kFlight];
#pragma unroll
    for (int q = 0; q < kFlight; ++q) {
      const size_t line = min(l0 + (size_t)q * kPersistThreads + tid, lines - 1);     // clamped: all loads issue together
      t[q] = ld_global(reinterpret_cast<const unsigned*>(base + line * 64));
    }
#pragma unroll
    for (int q = 0; q < kFlight; ++q) asm volatile("" ::"v"(t[q]));
  }
}

// The packed weight strips that XCD `x` will read in a GEMM phase with `n_tiles` strips in groups of NS and zg row
// groups (units in XCD-contiguous order), share `rank` of `count`.
__device__ __forceinline__ void persist_helper_weights(const half_t* Wp, int n_tiles, int K, int NS, int zg, int grid, int x,
                                                       int rank, int count) {
  const int n_units = ((n_tiles + NS - 1) / NS) * zg;
  if (n_units > grid) return;
  const int q = n_units >> 3, r = n_units & 7;
  const int lo = x * q + min(x, r), cnt = q + (x < r ? 1 : 0);
  if (cnt <= 0) return;
  const int s_lo = (lo / zg) * NS, s_hi = min(((lo + cnt - 1) / zg + 1) * NS, n_tiles);
  if (s_hi <= s_lo) return;
  const size_t strip = (size_t)K * 64, all = (size_t)(s_hi - s_lo) * strip;
  const size_t part = (all / count + 63) / 64 * 64, off = min(part * rank, all);
  persist_helper_touch(reinterpret_cast<const unsigned char*>(Wp) + (size_t)s_lo * strip + off, min(part, all - off));
}

// Waits (bounded) until the first pair of an exchange matrix carries this step's tag; false on give-up.  One wave
// polls for the workgroup (every polling wave is a request to the same address).
__device__ __forceinline__ bool persist_helper_wait(const unsigned char* buf, unsigned tag, unsigned limit, int* s_flag) {
  if (threadIdx.x < 64) {
    const __amdgpu_buffer_rsrc_t r = xch_rsrc(buf, 16);
    unsigned spins = 0;
    bool ok = true;
    while (true) {
      asm volatile("" ::: "memory");
      const u32x4 v = xch_load16(r, 0);
      if (v[1] == tag) break;
      if (++spins > limit) { ok = false; break; }
      __builtin_amdgcn_s_sleep(8);
    }
    if (threadIdx.x == 0) *s_flag = ok ? 1 : 0;
  }
  lds_barrier();
  const bool ok = *s_flag != 0;
  lds_barrier();          // the flag is free for the next wait
  return ok;
}

template <int RPW>
__device__ __forceinline__ void persist_helper(const PersistArgs& p, unsigned tag) {
  constexpr int R = 8 * RPW, R5 = 4 * RPW;
  const int grid = p.helpers_from;                 // workgroups that own units
  const int wg = blockIdx.x, x = wg & 7, rank = (wg - p.helpers_from) >> 3, count = ((int)gridDim.x - p.helpers_from) >> 3;
  const int d = p.d, f = p.f, B = p.B, H = p.H, S = p.S;
  const int zg = (B + R - 1) / R, zg5 = (B + R5 - 1) / R5;
  const int n_streams = B * H, rows = min(S, p.kv_rows);
  __shared__ int s_flag;
  const int lookahead = (p.dbg >> 4) ? (p.dbg >> 4) : 3;      // phases between a touch and its use (measurement hook: dbg / 16 overrides)
  for (int t = 0; t < 5 * p.n_layers; ++t) {
    const int l = t / 5, ph = t - 5 * l;
    if (t >= lookahead) {                          // stay `lookahead` phases ahead of the publishing front
      const int tw = t - lookahead, lw = tw / 5, pw = tw - 5 * lw;
      const unsigned char* xw = p.xch + (size_t)lw * p.xo.layer_bytes;
      const unsigned off = pw == 0 ? p.xo.qkv : pw == 1 ? p.xo.o : pw == 2 ? p.xo.y1 : pw == 3 ? p.xo.g : p.xo.y2;
      if (!persist_helper_wait(xw + off, tag, p.spin_limit, &s_flag)) return;
    }
    const PersistLayer L = p.layers[l];
    unsigned long long* tr = p.trace ? as_global(p.trace) + ((size_t)blockIdx.x * p.n_layers + l) * 32 : nullptr;
    persist_stamp(tr, 3 * ph);                     // tracing: the wait for the front ended
    if (ph == 0) persist_helper_weights(as_global(L.wqkv), 3 * d / 32, d, 2, zg, grid, x, rank, count);
    else if (ph == 2) persist_helper_weights(as_global(L.wo), d / 32, d, 1, zg, grid, x, rank, count);
    else if (ph == 3) persist_helper_weights(as_global(L.w1), f / 32, d, 2, zg, grid, x, rank, count);
    else if (ph == 4) persist_helper_weights(as_global(L.w2), d / 32, f, 1, zg5, grid, x, rank, count);
    else {
      // attention: unit u (streams 2u, 2u + 1) runs on workgroup u % grid; this XCD's units are those congruent
      // to x mod 8 (grid is a multiple of 8).  Items = (unit, stream, K | V), dealt round-robin to the helpers.
      const int n_units = (n_streams + 1) / 2;
      const int mine = (n_units - x + 7) / 8;      // units of this XCD
      for (int i = rank; i < mine * 4; i += count) {
        const int u = x + 8 * (i >> 2), s = 2 * u + ((i >> 1) & 1);
        if (s >= n_streams) continue;
        const int b = s / H, h = s - b * H;
        const int cb = p.slot ? p.slot[b] : b;
        const half_t* base = ((i & 1) ? as_global(L.vc) : as_global(L.kc)) + ((size_t)cb * H + h) * S * 64;
        persist_helper_touch(reinterpret_cast<const unsigned char*>(base), (size_t)rows * 128);
      }
    }
    persist_stamp(tr, 3 * ph + 2);                 // tracing: this phase's lines have arrived in the L2
  }
  // The projection kernel that follows on the stream reads strip s of the table in workgroup s, i.e. on XCD s mod 8:
  // with the last layer's operands in place, this XCD's helpers pull its strips (an eighth of the table, most of
  // what an L2 holds) while the others finish the layer.
  if (p.table_p && !(p.dbg & 4)) {
    const half_t* tp = as_global(p.table_p);
    const size_t strip = (size_t)d * 64;           // bytes
    for (int j = rank; x + 8 * j < p.table_strips; j += count)
      persist_helper_touch(reinterpret_cast<const unsigned char*>(tp) + (size_t)(x + 8 * j) * strip, strip);
  }
}

// RPW: rows per wave of the LayerNorm prologues (1 for B <= 32, 2 above); FRD / FR5: weight fragments per wave
// and strip in the GEMMs whose contraction is the model width / the FFN width (one per 128 of it); U: cache-row
// groups in flight per wave of the attention (a batch covers 32 U keys).
// Order inside a phase: request this phase's weight fragments, wait for the phase's input, compute, publish.
template <int RPW, int FRD, int FR5, int U>
__global__ __launch_bounds__(kPersistThreads) void decode_persist_kernel(PersistArgs p_in) {
  PersistArgs p = p_in;             // (pointers inside a by-value struct argument are not known to be global)
  p.layers = as_global(p.layers); p.tok = as_global(p.tok); p.cache_len = as_global(p.cache_len);
  p.tok_emb = as_global(p.tok_emb); p.pos_emb = as_global(p.pos_emb); p.seg_row = as_global(p.seg_row);
  p.emb_g = as_global(p.emb_g); p.emb_b = as_global(p.emb_b); p.finished = as_global(p.finished);
  p.slot = as_global(p.slot); p.xch = as_global(p.xch); p.epoch = as_global(p.epoch); p.X = as_global(p.X);
  p.hidden_out = as_global(p.hidden_out); p.err = as_global(p.err); p.trace = as_global(p.trace);
  p.table_p = as_global(p.table_p);
  extern __shared__ __align__(16) unsigned char smem_raw[];      // the A tile, then `red` behind it (p.red_off)
  __shared__ __align__(16) half_t sRes[16 * 32];
  __shared__ float sm[2][4][8][10];
  __shared__ int s_fail;
  if (threadIdx.x == 0) s_fail = 0;
  lds_barrier();
  float* red = reinterpret_cast<float*>(smem_raw + p.red_off);
  constexpr int R = 8 * RPW;        // rows per workgroup of the GEMM phases whose contraction is d
  constexpr int R5 = 4 * RPW;       // ... of the second FFN GEMM: its input row is four times as long
  const unsigned tag = *p.epoch + 1u;
  const int d = p.d, f = p.f, B = p.B;
  const int me = blockIdx.x;
  const int n_streams = B * p.H;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const bool no_w = (p.dbg & 2) != 0;
  if ((int)blockIdx.x >= p.helpers_from) {       // uniform for the workgroup
    if (!(p.dbg & 1)) persist_helper<RPW>(p, tag);
    return;
  }
  bool ok = true;
  // Weight fragments are requested at the start of their phase, before the wait for its input.  (Requesting them a
  // phase earlier, across the hand-over wait, needs two sets of fragments alive at once: up to 160 registers, which
  // the allocator answered with hundreds of spills -- and a spill reload waits for every outstanding load.)  The
  // helper workgroups have pulled them into this XCD's L2 by then.
  for (int l = 0; l < p.n_layers; ++l) {
    PersistLayer L = p.layers[l];
    L.wqkv = as_global(L.wqkv); L.wo = as_global(L.wo); L.w1 = as_global(L.w1); L.w2 = as_global(L.w2);
    L.bqkv = as_global(L.bqkv); L.bo = as_global(L.bo); L.b1 = as_global(L.b1); L.b2 = as_global(L.b2);
    L.ln1_g = as_global(L.ln1_g); L.ln1_b = as_global(L.ln1_b); L.ln2_g = as_global(L.ln2_g); L.ln2_b = as_global(L.ln2_b);
    L.kc = as_global(L.kc); L.vc = as_global(L.vc);
    unsigned char* xl = p.xch + (size_t)l * p.xo.layer_bytes;
    const bool hook = l == 0;
    unsigned long long* tr = p.trace ? p.trace + ((size_t)blockIdx.x * p.n_layers + l) * 32 : nullptr;
    persist_stamp(tr, 0);
    unsigned owned = 0;
    if (tr && l == 0 && threadIdx.x == 0) tr[15] = clock64();      // shader clock at the start (slot 15 of layer 0)
    {  // phase 1: QKV = LayerNorm(previous layer's sum, or the embedding) x Wqkv^T + bqkv
      PersistGemm g{};
      g.Wp = L.wqkv; g.N = 3 * d; g.K = d; g.B = B; g.eps = p.eps;
      g.xout = xl + p.xo.x; g.bias = L.bqkv; g.out = xl + p.xo.qkv; g.withhold = hook && p.stall == 1;
      PersistW<2, FRD> w_qkv;
      persist_w_issue<R, 2, FRD>(w_qkv, L.wqkv, 3 * d, d, B, no_w);
      const PersistUnit<R, 2> un = persist_unit<R, 2>(3 * d, B, L.bqkv);
      if (un.has) owned |= 1u;
      if (l == 0) {
        g.gamma = p.emb_g; g.beta = p.emb_b;
        ok = persist_gemm_in<R, 2, PRO_EMBED, PEPI_BIAS>(g, p, tag, smem_raw, sRes, &s_fail, un);
      } else {
        const PersistLayer P = p.layers[l - 1];
        g.in = xl - p.xo.layer_bytes + p.xo.y2; g.gamma = as_global(P.ln2_g); g.beta = as_global(P.ln2_b);
        ok = persist_gemm_in<R, 2, PRO_LN, PEPI_BIAS>(g, p, tag, smem_raw, sRes, &s_fail, un);
      }
      if (!ok) break;
      persist_stamp(tr, 1);
      persist_gemm_out<R, 2, FRD, PEPI_BIAS>(g, tag, smem_raw, red, sRes, un, w_qkv, tr, 16);
    }
    persist_stamp(tr, 2); persist_stamp(tr, 3);
    {  // phase 2: attention over the cache
      const __amdgpu_buffer_rsrc_t r_qkv = xch_rsrc(xl + p.xo.qkv, (unsigned)B * 3 * d * 4);
      PersistKV<U> kv;
      if (p.attn_nt) persist_kv_issue<U, true>(kv, p, L, me); else persist_kv_issue<U, false>(kv, p, L, me);
      PersistQKV x;
      bool good = true;
      {
        const int s = me * 2 + (wave >> 2);
        const int sc = min(s, n_streams - 1), b = sc / p.H, h = sc - b * p.H;
        const bool done = p.eos >= 0 && (p.finished[b] != 0 || p.tok[b] == p.eos);
        if (s < n_streams && !done) good = persist_qkv_wait(x, p, r_qkv, b, h, tag);
      }
      persist_stamp(tr, 4);
      const bool wh = hook && p.stall == 2;
      if (me * 2 < n_streams) owned |= 2u;
      if (me * 2 < n_streams)
        ok = p.attn_nt ? persist_attn_pair<U, true>(p, L, xl, tag, wh, me, kv, true, x, true, good, sm, &s_fail, tr)
                       : persist_attn_pair<U, false>(p, L, xl, tag, wh, me, kv, true, x, true, good, sm, &s_fail, tr);
      for (int u0 = me + p.helpers_from; ok && u0 * 2 < n_streams; u0 += p.helpers_from)
        ok = p.attn_nt ? persist_attn_pair<U, true>(p, L, xl, tag, wh, u0, kv, false, x, false, true, sm, &s_fail)
                       : persist_attn_pair<U, false>(p, L, xl, tag, wh, u0, kv, false, x, false, true, sm, &s_fail);
      if (!ok) break;
    }
    persist_stamp(tr, 5); persist_stamp(tr, 6);
    {  // phase 3: y1 = O x Wo^T + bo + x
      PersistGemm g{};
      g.Wp = L.wo; g.N = d; g.K = d; g.B = B; g.in = xl + p.xo.o; g.bias = L.bo; g.res = xl + p.xo.x;
      g.out = xl + p.xo.y1; g.withhold = hook && p.stall == 3;
      PersistW<1, FRD> w_o;
      persist_w_issue<R, 1, FRD>(w_o, L.wo, d, d, B, no_w);
      const PersistUnit<R, 1> un = persist_unit<R, 1>(d, B, L.bo);
      if (un.has) owned |= 4u;
      ok = persist_gemm_in<R, 1, PRO_COPY, PEPI_RES, RPW * FRD / 2>(g, p, tag, smem_raw, sRes, &s_fail, un);
      if (!ok) break;
      persist_stamp(tr, 7);
      persist_gemm_out<R, 1, FRD, PEPI_RES>(g, tag, smem_raw, red, sRes, un, w_o);
    }
    persist_stamp(tr, 8); persist_stamp(tr, 9);
    {  // phase 4: G = gelu(LayerNorm(y1) x W1^T + b1)
      PersistGemm g{};
      g.Wp = L.w1; g.N = f; g.K = d; g.B = B; g.eps = p.eps; g.in = xl + p.xo.y1; g.gamma = L.ln1_g; g.beta = L.ln1_b;
      g.xout = xl + p.xo.x1; g.bias = L.b1; g.out = xl + p.xo.g; g.withhold = hook && p.stall == 4;
      PersistW<2, FRD> w_1;
      persist_w_issue<R, 2, FRD>(w_1, L.w1, f, d, B, no_w);
      const PersistUnit<R, 2> un = persist_unit<R, 2>(f, B, L.b1);
      if (un.has) owned |= 8u;
      ok = persist_gemm_in<R, 2, PRO_LN, PEPI_GELU>(g, p, tag, smem_raw, sRes, &s_fail, un);
      if (!ok) break;
      persist_stamp(tr, 10);
      persist_gemm_out<R, 2, FRD, PEPI_GELU>(g, tag, smem_raw, red, sRes, un, w_1, tr, 20);
    }
    persist_stamp(tr, 11); persist_stamp(tr, 12);
    {  // phase 5: y2 = G x W2^T + b2 + x1
      PersistGemm g{};
      g.Wp = L.w2; g.N = d; g.K = f; g.B = B; g.in = xl + p.xo.g; g.bias = L.b2; g.res = xl + p.xo.x1;
      g.out = xl + p.xo.y2; g.withhold = hook && p.stall == 5;
      PersistW<1, FR5> w_2;
      persist_w_issue<R5, 1, FR5>(w_2, L.w2, d, f, B, no_w);
      const PersistUnit<R5, 1> un = persist_unit<R5, 1>(d, B, L.b2);
      if (un.has) owned |= 16u;
      ok = persist_gemm_in<R5, 1, PRO_COPY, PEPI_RES, RPW * FR5 / 4>(g, p, tag, smem_raw, sRes, &s_fail, un);
      if (!ok) break;
      persist_stamp(tr, 13);
      persist_gemm_out<R5, 1, FR5, PEPI_RES>(g, tag, smem_raw, red, sRes, un, w_2, tr, 24);
    }
    persist_stamp(tr, 14);
    if (tr && threadIdx.x == 0) tr[31] = owned;      // tracing: the phases (bit 0 = QKV .. bit 4 = FFN2) this workgroup owned a unit of
  }
  if (ok) {
    const int last = p.n_layers - 1;
    PersistLayer L = p.layers[last];
    L.ln2_g = as_global(L.ln2_g); L.ln2_b = as_global(L.ln2_b);
    ok = persist_final_ln<2>(p, L, p.xch + (size_t)last * p.xo.layer_bytes + p.xo.y2, tag, &s_fail);
  }
  if (p.trace && threadIdx.x == 0) {       // shader-clock reading next to the last 100 MHz stamp: slot 15 of the last layer
    unsigned long long* row = p.trace + ((size_t)blockIdx.x * p.n_layers + (p.n_layers - 1)) * 32;
    row[15] = clock64();
  }
  if (!ok && threadIdx.x == 0) *p.err = 1;
}

// Advances the step counter of the hand-over tags; launched after the persistent kernel on the same stream.
__global__ void persist_epoch_bump_kernel(unsigned* epoch) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *epoch += 1u;
}

}  // namespace ernie
