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
// phase are requested before the workgroup starts polling for the phase's input, so the HBM stream runs
// under the hand-over latency.  Row-wise work sits where the full row is: LayerNorm in the prologue of the
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
};

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

enum { PRO_LN = 0, PRO_EMBED = 1, PRO_COPY = 2 };
enum { PEPI_BIAS = 0, PEPI_RES = 1, PEPI_GELU = 2 };

struct PersistGemm {
  const half_t* Wp; int N, K, B;
  const unsigned char* in; const float* gamma; const float* beta; float eps;     // prologue
  unsigned char* xout;                 // PRO_LN / PRO_EMBED: normalised rows as pairs (written by strip group 0)
  const float* bias;                   // [N]
  const unsigned char* res;            // PEPI_RES: residual rows [B][N] as pairs
  unsigned char* out;                  // [B][N] as pairs
  bool withhold;                       // test hook: compute, but do not publish
};

// One GEMM-shaped phase.  R rows per workgroup (PRO_LN / PRO_EMBED: one or two rows per wave, R = 8 or 16),
// NS strips per workgroup, FR weight fragments in flight per wave and strip.  Returns false (uniformly for the
// workgroup) when a wait gave up.
template <int R, int NS, int FR, int PRO, int EPI, int RC = 2>
__device__ __forceinline__ bool persist_gemm_phase(const PersistGemm& g, const PersistArgs& p, unsigned tag,
                                                   unsigned char* smem_raw) {
  constexpr int NW = kPersistWaves;
  constexpr int NV = R <= 8 ? 4 : R / 2;      // accumulator registers that hold rows < R (row = 8 (v / 4) + 4 (lane / 32) + v % 4)
  constexpr int RPW = R / NW;                 // LayerNorm prologues: rows per wave
  static_assert(PRO == PRO_COPY || R == 8 || R == 16, "LayerNorm prologue: one or two rows per wave");
  static_assert(EPI != PEPI_RES || NS == 1, "the residual tile is one strip wide");
  __shared__ __align__(16) half_t sRes[16 * 32];
  half_t* sA = reinterpret_cast<half_t*>(smem_raw);            // [R][K + 8]
  float* red = reinterpret_cast<float*>(smem_raw);             // [NW][NS * NV][64], reused after the MFMA loop

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = g.K, B = g.B, N = g.N;
  const int k_tiles = K / 16, n_tiles = N / 32, pitch = K + 8;
  const int kb = k_tiles * wave / NW, ke = k_tiles * (wave + 1) / NW;
  const int zg = (B + R - 1) / R, sgs = (n_tiles + NS - 1) / NS, n_units = sgs * zg;
  const __amdgpu_buffer_rsrc_t r_in = xch_rsrc(g.in, (unsigned)B * K * 4);
  const __amdgpu_buffer_rsrc_t r_out = xch_rsrc(g.out, (unsigned)B * N * 4);
  const __amdgpu_buffer_rsrc_t r_xout = xch_rsrc(g.xout, (unsigned)B * K * 4);
  const __amdgpu_buffer_rsrc_t r_res = xch_rsrc(g.res, (unsigned)B * N * 4);

  for (int u0 = blockIdx.x; u0 < n_units; u0 += gridDim.x) {
    // XCD-contiguous order, row group fastest: the row groups of a strip group run on one XCD and share its
    // weight fragments in that L2
    const int logical = n_units <= (int)gridDim.x ? xcd_contiguous_id(u0, n_units) : u0;
    const int sg = logical / zg, zi = logical - sg * zg;
    const int row0 = zi * R;

    // 1. weight stream first: it runs under the wait for this phase's input
    const half_t* wp[NS];
    half8 wf[NS][FR];
#pragma unroll
    for (int n = 0; n < NS; ++n) {
      wp[n] = g.Wp + packed_frag_offset(min(sg * NS + n, n_tiles - 1), 0, k_tiles) + lane * 8;
#pragma unroll
      for (int u = 0; u < FR; ++u)
        wf[n][u] = *reinterpret_cast<const half8*>(wp[n] + (size_t)min(kb + u, k_tiles - 1) * 512);
    }

    // the bias of this lane's output columns travels with the weights (the epilogue would otherwise start with a
    // memory round trip of its own)
    constexpr int kMyNv = (NS * NV + NW - 1) / NW;
    float bias_r[kMyNv];
#pragma unroll
    for (int i = 0; i < kMyNv; ++i) {
      const int nt = sg * NS + (wave + i * NW) / NV;
      bias_r[i] = g.bias[min(nt * 32 + (lane & 31), N - 1)];
    }

    bool fail = false;
    // 2. prologue: the A tile [R][K] as fp16 in LDS
    if constexpr (PRO == PRO_COPY) {
      const int upr = K / 4;                         // 16-byte units (4 values) per row
      const int total = R * upr;
      constexpr int kPieces = 4;
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
          const int id = min(id0 + q * kPersistThreads, total - 1);     // clamped: a duplicate is loaded, not stored
          const int r = id / upr, c4 = id - r * upr;
          off[q] = ((unsigned)min(row0 + r, B - 1) * K + c4 * 4) * 4;
          dst[q] = r * pitch + c4 * 4;
        }
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
        const float4 g0 = *reinterpret_cast<const float4*>(g.gamma + cc * 8), g1 = *reinterpret_cast<const float4*>(g.gamma + cc * 8 + 4);
        const float4 t0 = *reinterpret_cast<const float4*>(g.beta + cc * 8), t1 = *reinterpret_cast<const float4*>(g.beta + cc * 8 + 4);
        gm[c][0] = g0.x; gm[c][1] = g0.y; gm[c][2] = g0.z; gm[c][3] = g0.w; gm[c][4] = g1.x; gm[c][5] = g1.y; gm[c][6] = g1.z; gm[c][7] = g1.w;
        bt[c][0] = t0.x; bt[c][1] = t0.y; bt[c][2] = t0.z; bt[c][3] = t0.w; bt[c][4] = t1.x; bt[c][5] = t1.y; bt[c][6] = t1.z; bt[c][7] = t1.w;
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
            const half8 e = *reinterpret_cast<const half8*>(p.tok_emb + (size_t)id * K + cc * 8);
            const half8 q = *reinterpret_cast<const half8*>(p.pos_emb + (size_t)pos * K + cc * 8);
            half8 s8 = {0, 0, 0, 0, 0, 0, 0, 0};
            if (p.seg_row) s8 = *reinterpret_cast<const half8*>(p.seg_row + cc * 8);
            const float live = (c * 64 + lane < chunks) ? 1.f : 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[i][c][j] = ((float)e[j] + (float)q[j] + (float)s8[j]) * live;
          }
        }
      } else {
        u32x4 a[RPW][RC][2];
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
      for (int o = 32; o > 0; o >>= 1)
#pragma unroll
        for (int i = 0; i < RPW; ++i) mean[i] += __shfl_xor(mean[i], o, 64);
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
      for (int o = 32; o > 0; o >>= 1)
#pragma unroll
        for (int i = 0; i < RPW; ++i) rstd[i] += __shfl_xor(rstd[i], o, 64);
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        const int r = row0 + wave * RPW + i;
        const float rs = rsqrtf(rstd[i] / (float)K + g.eps);
        const bool writer = sg == 0 && r < B && !fail;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
          const int ch = c * 64 + lane;
          if (ch < chunks) {
            half8 o;
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = (half_t)((v[i][c][j] - mean[i]) * rs * gm[c][j] + bt[c][j]);
            *reinterpret_cast<half8*>(sA + (wave * RPW + i) * pitch + ch * 8) = o;
            if (writer) {
              const u32x4 w = __builtin_bit_cast(u32x4, o);
              const unsigned off = ((unsigned)r * K + ch * 8) * 4;
              xch_store16(r_xout, off, w[0], w[1], tag);
              xch_store16(r_xout, off + 16, w[2], w[3], tag);
            }
          }
        }
      }
    }
    if (__syncthreads_or(fail)) return false;

    // 3. MFMA over this wave's k-tiles
    floatx16 acc[NS];
#pragma unroll
    for (int n = 0; n < NS; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    const half_t* ap = sA + (lane & (R - 1)) * pitch + 8 * (lane >> 5);    // tile rows R..31 repeat rows 0..R-1
    for (int base = kb; base < ke; base += FR) {
#pragma unroll
      for (int u = 0; u < FR; ++u)
        if (base + u < ke) {
          const half8 a = *reinterpret_cast<const half8*>(ap + (base + u) * 16);
#pragma unroll
          for (int n = 0; n < NS; ++n) acc[n] = mfma32(a, wf[n][u], acc[n]);
        }
      if (base + FR < ke) {
#pragma unroll
        for (int n = 0; n < NS; ++n)
#pragma unroll
          for (int u = 0; u < FR; ++u)
            wf[n][u] = *reinterpret_cast<const half8*>(wp[n] + (size_t)min(base + FR + u, k_tiles - 1) * 512);
      }
    }
    __syncthreads();          // all waves are done reading sA before it is reused

    // 4. cross-wave reduction in a fixed order, then the epilogue
#pragma unroll
    for (int n = 0; n < NS; ++n)
#pragma unroll
      for (int v = 0; v < NV; ++v) red[(wave * NS * NV + n * NV + v) * 64 + lane] = acc[n][v];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kMyNv; ++i) {
      const int nv = wave + i * NW;
      if (nv >= NS * NV) break;
      const int n = nv / NV, v = nv - n * NV;
      const int nt = sg * NS + n;
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += red[(w * NS * NV + nv) * 64 + lane];
      const int tr = mfma32_row(v, lane);                 // row inside the tile
      const int row = row0 + tr, col = nt * 32 + (lane & 31);
      const bool live = nt < n_tiles && tr < R && row < B;
      float val = s + bias_r[i];
      if constexpr (EPI == PEPI_RES) val += (float)sRes[min(tr, R - 1) * 32 + (lane & 31)];
      if constexpr (EPI == PEPI_GELU) val = gelu_erf_fast(val);
      const float nb = __shfl_xor(val, 1, 64);            // the odd neighbour column
      if (live && (lane & 1) == 0 && !g.withhold)
        xch_store8(r_out, ((unsigned)row * N + col) * 4, pack_h2(val, nb), tag);
    }
    __syncthreads();          // `red` / `sRes` are free for the next unit or phase
  }
  return true;
}

// Decode attention of one layer: a group of four waves per (sequence, head) stream, two streams per
// workgroup at a time.  q, k, v of the new token come from the exchange buffer (QKV output + bias, already
// fp16); the new key and value are appended to the cache and used from registers.  The first batch of cache
// rows is requested before the wait for q, k, v.
template <int U, bool NT>
__device__ __forceinline__ bool persist_attn_phase(const PersistArgs& p, const PersistLayer& L, unsigned char* xl,
                                                   unsigned tag, bool withhold) {
  constexpr int NW = 4;
  __shared__ float sm[2][NW][8][10];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, w4 = wave & 3;
  const int ec = lane & 7, team = lane >> 3;
  const int B = p.B, H = p.H, S = p.S, d = p.d;
  const int n_streams = B * H;
  const __amdgpu_buffer_rsrc_t r_qkv = xch_rsrc(xl + p.xo.qkv, (unsigned)B * 3 * d * 4);
  const __amdgpu_buffer_rsrc_t r_o = xch_rsrc(xl + p.xo.o, (unsigned)B * d * 4);

  for (int u0 = blockIdx.x; u0 * 2 < n_streams; u0 += gridDim.x) {
    const int s = u0 * 2 + grp;
    const bool active = s < n_streams;
    const int b = active ? s / H : 0, h = active ? s - b * H : 0;
    // a sequence that is fed the end token (now or at an earlier step) is finished: no cache stream, no append
    const bool done = active && p.eos >= 0 && (p.finished[b] != 0 || p.tok[b] == p.eos);
    bool fail = false;
    SoftmaxPart st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j] = 0.f;

    if (active && !done) {
      const int cb = p.slot ? p.slot[b] : b;
      half_t* Kb = L.kc + ((size_t)cb * H + h) * S * 64 + ec * 8;
      half_t* Vb = L.vc + ((size_t)cb * H + h) * S * 64 + ec * 8;
      half8 kf[U], vf[U];
      int key[U];
      int g0 = w4 * U;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        key[u] = (g0 + u) * 8 + team;
        const size_t row = (size_t)min(key[u], S - 1) * 64;
        kf[u] = load_kv<NT>(Kb + row);
        vf[u] = load_kv<NT>(Vb + row);
      }
      const int len = p.cache_len[b];

      float q[8];
      half8 knew, vnew;
      {
        const unsigned off = ((unsigned)b * 3 * d + h * 64 + ec * 8) * 4;
        u32x4 a[3][2];
        unsigned spins = 0;
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
          if (++spins > p.spin_limit) { fail = true; break; }
        }
        float qq[8];
        unpack_h2(a[0][0][0], qq[0], qq[1]); unpack_h2(a[0][0][2], qq[2], qq[3]);
        unpack_h2(a[0][1][0], qq[4], qq[5]); unpack_h2(a[0][1][2], qq[6], qq[7]);
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = qq[j] * 0.125f;
        const u32x4 kw = {a[1][0][0], a[1][0][2], a[1][1][0], a[1][1][2]};
        const u32x4 vw = {a[2][0][0], a[2][0][2], a[2][1][0], a[2][1][2]};
        knew = __builtin_bit_cast(half8, kw);
        vnew = __builtin_bit_cast(half8, vw);
      }
      const bool has_new = len < S;                 // a replayed step past capacity appends nothing
      const int c = fail ? 0 : (has_new ? len + 1 : S);
      const int newest = has_new ? len : -1;        // this key comes from registers, not from the cache
      if (!fail && has_new && w4 == 0 && team == 0) {
        *reinterpret_cast<half8*>(Kb + (size_t)len * 64) = knew;
        *reinterpret_cast<half8*>(Vb + (size_t)len * 64) = vnew;
      }
      while (g0 * 8 < c) {
        float sc[U];
        float mx = st.m;
        half8 vcur[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const bool valid = key[u] < c;
          const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
          if (key[u] == newest) { kf[u] = knew; vf[u] = vnew; }
          float pr = 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) pr += q[j] * (float)kf[u][j];
          pr += __shfl_xor(pr, 1, 64);
          pr += __shfl_xor(pr, 2, 64);
          pr += __shfl_xor(pr, 4, 64);
          sc[u] = valid ? pr : -INFINITY;
          vcur[u] = valid ? vf[u] : z;
          mx = fmaxf(mx, sc[u]);
        }
        g0 += NW * U;
        if (g0 * 8 < c) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            key[u] = (g0 + u) * 8 + team;
            const size_t row = (size_t)min(key[u], S - 1) * 64;
            kf[u] = load_kv<NT>(Kb + row);
            vf[u] = load_kv<NT>(Vb + row);
          }
        }
        if (mx != -INFINITY) {
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
          st.m = mx;
        }
      }
#pragma unroll
      for (int off = 8; off < 64; off <<= 1) {
        const float om = __shfl_xor(st.m, off, 64);
        const float ol = __shfl_xor(st.l, off, 64);
        float oa[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) oa[j] = __shfl_xor(st.acc[j], off, 64);
        softmax_merge(st, om, ol, oa);
      }
      if (team == 0) {
        sm[grp][w4][ec][0] = st.m; sm[grp][w4][ec][1] = st.l;
#pragma unroll
        for (int j = 0; j < 8; ++j) sm[grp][w4][ec][2 + j] = st.acc[j];
      }
    }
    if (__syncthreads_or(fail)) return false;
    if (active && w4 == 0 && team == 0) {
      float o8[8];
      if (done) {
#pragma unroll
        for (int j = 0; j < 8; ++j) o8[j] = 0.f;          // the row is not used; its consumers still need the tag
      } else {
#pragma unroll
        for (int w = 1; w < NW; ++w) softmax_merge(st, sm[grp][w][ec][0], sm[grp][w][ec][1], &sm[grp][w][ec][2]);
        const float inv = 1.0f / st.l;
#pragma unroll
        for (int j = 0; j < 8; ++j) o8[j] = st.acc[j] * inv;
      }
      if (!withhold) {
        const unsigned off = ((unsigned)b * d + h * 64 + ec * 8) * 4;
        xch_store16(r_o, off, pack_h2(o8[0], o8[1]), pack_h2(o8[2], o8[3]), tag);
        xch_store16(r_o, off + 16, pack_h2(o8[4], o8[5]), pack_h2(o8[6], o8[7]), tag);
      }
    }
    __syncthreads();          // `sm` is free for the next pair of streams
  }
  return true;
}

// Final LayerNorm of the step: one wave per row reads the last layer's pre-LayerNorm sums from the exchange
// buffer and writes the plain fp16 rows the projection kernel reads (and the caller's fp32 copy).
template <int RC>
__device__ __forceinline__ bool persist_final_ln(const PersistArgs& p, const PersistLayer& L, const unsigned char* y2,
                                                 unsigned tag) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int d = p.d, B = p.B, chunks = d / 8;
  const __amdgpu_buffer_rsrc_t r_in = xch_rsrc(y2, (unsigned)B * d * 4);
  bool fail = false;
  for (int r = blockIdx.x * kPersistWaves + wave; r < B; r += gridDim.x * kPersistWaves) {
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
  return !__syncthreads_or(fail);
}

// RPW: rows per wave of the LayerNorm prologues (1 for B <= 32, 2 above); FR5: weight fragments in flight per
// wave in the second FFN GEMM, whose contraction is the FFN width (8 per 1024 of it).
template <int RPW, int FR5>
__global__ __launch_bounds__(kPersistThreads) void decode_persist_kernel(PersistArgs p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  constexpr int R = 8 * RPW;        // rows per workgroup of the GEMM phases whose contraction is d
  constexpr int R5 = 4 * RPW;       // ... of the second FFN GEMM: its input row is four times as long
  const unsigned tag = *p.epoch + 1u;
  const int d = p.d, f = p.f, B = p.B;
  bool ok = true;
  for (int l = 0; l < p.n_layers && ok; ++l) {
    const PersistLayer L = p.layers[l];
    unsigned char* xl = p.xch + (size_t)l * p.xo.layer_bytes;
    const bool hook = l == 0;
    {  // phase 1: QKV = LayerNorm(previous layer's sum, or the embedding) x Wqkv^T + bqkv
      PersistGemm g{};
      g.Wp = L.wqkv; g.N = 3 * d; g.K = d; g.B = B; g.eps = p.eps;
      g.xout = xl + p.xo.x; g.bias = L.bqkv; g.out = xl + p.xo.qkv; g.withhold = hook && p.stall == 1;
      if (l == 0) {
        g.gamma = p.emb_g; g.beta = p.emb_b;
        ok = persist_gemm_phase<R, 2, 8, PRO_EMBED, PEPI_BIAS>(g, p, tag, smem_raw);
      } else {
        const PersistLayer P = p.layers[l - 1];
        g.in = xl - p.xo.layer_bytes + p.xo.y2; g.gamma = P.ln2_g; g.beta = P.ln2_b;
        ok = persist_gemm_phase<R, 2, 8, PRO_LN, PEPI_BIAS>(g, p, tag, smem_raw);
      }
    }
    if (!ok) break;
    // phase 2: attention over the cache
    ok = p.attn_nt ? persist_attn_phase<4, true>(p, L, xl, tag, hook && p.stall == 2)
                   : persist_attn_phase<4, false>(p, L, xl, tag, hook && p.stall == 2);
    if (!ok) break;
    {  // phase 3: y1 = O x Wo^T + bo + x
      PersistGemm g{};
      g.Wp = L.wo; g.N = d; g.K = d; g.B = B; g.in = xl + p.xo.o; g.bias = L.bo; g.res = xl + p.xo.x;
      g.out = xl + p.xo.y1; g.withhold = hook && p.stall == 3;
      ok = persist_gemm_phase<R, 1, 8, PRO_COPY, PEPI_RES>(g, p, tag, smem_raw);
    }
    if (!ok) break;
    {  // phase 4: G = gelu(LayerNorm(y1) x W1^T + b1)
      PersistGemm g{};
      g.Wp = L.w1; g.N = f; g.K = d; g.B = B; g.eps = p.eps; g.in = xl + p.xo.y1; g.gamma = L.ln1_g; g.beta = L.ln1_b;
      g.xout = xl + p.xo.x1; g.bias = L.b1; g.out = xl + p.xo.g; g.withhold = hook && p.stall == 4;
      ok = persist_gemm_phase<R, 2, 8, PRO_LN, PEPI_GELU>(g, p, tag, smem_raw);
    }
    if (!ok) break;
    {  // phase 5: y2 = G x W2^T + b2 + x1
      PersistGemm g{};
      g.Wp = L.w2; g.N = d; g.K = f; g.B = B; g.in = xl + p.xo.g; g.bias = L.b2; g.res = xl + p.xo.x1;
      g.out = xl + p.xo.y2; g.withhold = hook && p.stall == 5;
      ok = persist_gemm_phase<R5, 1, FR5, PRO_COPY, PEPI_RES>(g, p, tag, smem_raw);
    }
  }
  if (ok) {
    const int last = p.n_layers - 1;
    ok = persist_final_ln<2>(p, p.layers[last], p.xch + (size_t)last * p.xo.layer_bytes + p.xo.y2, tag);
  }
  if (!ok && threadIdx.x == 0) *p.err = 1;
}

// Advances the step counter of the hand-over tags; launched after the persistent kernel on the same stream.
__global__ void persist_epoch_bump_kernel(unsigned* epoch) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *epoch += 1u;
}

}  // namespace ernie
