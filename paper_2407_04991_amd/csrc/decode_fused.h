// Latency-oriented decode-step kernels for small batches (B <= 64).
//
// At B = 32 one decode step moves only 1-5 MB per GEMM, so a step is bound by
// the number of dependent phases, not by any single kernel.  These kernels cut
// a layer to five phases by moving every row-wise operation into the PROLOGUE
// of its consumer:
//
//   gemm_dec_ln   A = LayerNorm(sum_k partial_k + bias + residual)     (QKV, FFN1)
//   gemm_dec      A = fp16 activations                                 (out-proj, FFN2, logits)
//   attn_decode_fused   q, k, v = raw + bias; append k, v; attend            (attention)
//
// A GEMM phase writes raw fp32 accumulators (optionally split over K into
// `gridDim.y` partial buffers that the consumer adds in a fixed order), so the
// result does not depend on scheduling; FFN1 instead applies bias + GELU in its
// epilogue, where every element is computed exactly once.  Each workgroup issues its weight
// fragment loads BEFORE the prologue: the HBM latency of the weight stream
// hides under the L2-resident activation work.
#pragma once

#include <type_traits>

#include "common.h"
#include "rowops.h"

namespace ernie {

enum { EPI_RAW = 0, EPI_ARGMAX = 1, EPI_GELU16 = 2 };

constexpr int kDecMaxFrag = 8;   // weight fragments a wave keeps in flight

struct DecGemmArgs {
  const half_t* Wp;   // packed [N, K]
  int N, K, B;
  // prologue inputs
  const half_t* a16;  // gemm_dec: [B, K] fp16
  const float* r32;   // gemm_dec_ln: raw fp32 [sk_in][B][K]
  int sk_in;
  const float* bias;  // [K] bias of the GEMM that produced r32
  const half_t* res;  // gemm_dec_ln: residual [B, K] fp16
  const float* gamma;
  const float* beta;
  float eps;
  half_t* xout;       // gemm_dec_ln: normalised rows [B, K] fp16, written by the strip-0 workgroups; may be null
  // gemm_dec_ln with SKIN = 0 (embedding prologue): A = LayerNorm(E'[tok[b]] + Epos[len[b]] (+ segment row))
  const int* tok;         // [B] ids fed to this step
  const int* cache_len;   // [B] position of the new token
  const half_t* tok_emb;  // [V', K] row-major trimmed table
  const half_t* pos_emb;  // [P, K]
  const half_t* seg_row;  // [K] or null
  int max_pos;
  int vocab_kept;         // rows of tok_emb: fed ids are clamped into the table
  int eos;                // >= 0: a row fed this id is marked finished (by the strip-0 workgroups)
  int* finished;
  // outputs
  float* rout;        // EPI_RAW: [gridDim.y][B][N]
  const float* bias_out;  // EPI_GELU16: [N] bias of THIS GEMM; EPI_ARGMAX: optional [N] output bias (may be null)
  half_t* g16;        // EPI_GELU16: gelu(acc + bias_out) as fp16 [B, N]; needs gridDim.y == 1
  float* logits_out;  // EPI_ARGMAX: [B, N] or null
  float* strip_val;   // EPI_ARGMAX: [B, strips]
  int* strip_idx;
  int strips;
  // gemm_dec: workgroups with blockIdx.x >= n_main only warm the L2 for the next kernel
  int n_main;
  DecPrefetch pf;
  KvPrefetch kv;      // warming workgroups past pf.count stream the next attention's cache rows
};

// Shared epilogue of the decode GEMMs: `s` is the finished accumulator of (row, col).
template <int EPI>
__device__ __forceinline__ void dec_epilogue(const DecGemmArgs& p, int nt, int lane, int row, int col, float s) {
  const int B = p.B;
  if constexpr (EPI == EPI_RAW) {
    if (row < B && col < p.N) p.rout[((size_t)blockIdx.y * B + row) * p.N + col] = s;
  } else if constexpr (EPI == EPI_GELU16) {
    if (row < B && col < p.N) p.g16[(size_t)row * p.N + col] = (half_t)gelu_erf_fast(s + p.bias_out[col]);
  } else {
    if (p.bias_out && col < p.N) s += p.bias_out[col];      // optional output bias of the projection
    if (p.logits_out && row < B && col < p.N) p.logits_out[(size_t)row * p.N + col] = s;
    float bv = (col < p.N) ? s : -INFINITY;      // best of this strip for `row`: reduce over the 32 lanes of a half-wave
    int bi = col;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      argmax_merge(bv, bi, ov, oi);
    }
    if ((lane & 31) == 0 && row < B) {
      p.strip_val[(size_t)row * p.strips + nt] = bv;
      p.strip_idx[(size_t)row * p.strips + nt] = bi;
    }
  }
}

// A = fp16 activations [B, K].  grid = (column strips, split-K); MT = ceil(B / 32) row tiles.
template <int MT, int NW, int EPI>
__global__ __launch_bounds__(NW * 64) void gemm_dec_kernel(DecGemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* sA = reinterpret_cast<half_t*>(smem_raw);
  float* red = reinterpret_cast<float*>(smem_raw);   // reused after the MFMA loop

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int nt = blockIdx.x;
  if (nt >= p.n_main) {      // uniform for the workgroup
    const int idx = (nt - p.n_main) + (gridDim.x - p.n_main) * blockIdx.y;
    const int wg_id = nt + gridDim.x * blockIdx.y;
    if (idx < p.pf.count) dec_prefetch_run(p.pf, idx, wg_id, tid, NW * 64);
    else kv_prefetch_run(p.kv, idx - p.pf.count, wg_id, tid, NW * 64);
    return;
  }
  const int K = p.K, B = p.B;
  const int k_tiles = K / 16;
  const int tiles_wg = k_tiles / gridDim.y;           // host guarantees divisibility
  const int tile0 = blockIdx.y * tiles_wg;
  const int kslice = tiles_wg * 16, k0 = tile0 * 16;
  const int pitch = kslice + 8;
  const int kb = tiles_wg * wave / NW, ke = tiles_wg * (wave + 1) / NW;

  // 1. weight stream: first batch of fragments in flight before anything else
  const half_t* wp = p.Wp + packed_frag_offset(nt, tile0, k_tiles) + lane * 8;
  half8 wf[kDecMaxFrag];
#pragma unroll
  for (int u = 0; u < kDecMaxFrag; ++u) {
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    wf[u] = (kb + u < ke) ? *reinterpret_cast<const half8*>(wp + (size_t)(kb + u) * 512) : z;
  }

  // 2. prologue: copy the fp16 A tile [MT * 32, kslice] into LDS (rows >= B re-read row B-1; their
  //    products land in accumulator rows that are never stored)
  //    All pieces of a thread (up to eight 16-byte pieces per batch) are requested together, and the first
  //    batch, which covers the whole tile at the usual sizes, is straight-line code with exactly as many
  //    pieces as the tile needs: a loop of one load and one LDS store per trip spends a memory round trip per
  //    trip, and the compiler drains all outstanding loads (the weight stream above) at a loop header.
  //    Pieces past the end wrap around (spread over the tile, not piled on one address) and are not stored.
  {
    const int chunks = kslice / 8;
    const int total = MT * 32 * chunks;
    // piece id -> (row, chunk) by stepping: one division per batch instead of one per piece (the divisions were
    // a fifth of this kernel's code)
    const int step_r = (NW * 64) / chunks, step_c = (NW * 64) - step_r * chunks;
    auto copy_batch = [&](int id0, auto pieces_tag) {
      constexpr int kPieces = decltype(pieces_tag)::value;
      half8 v[kPieces];
      int dst[kPieces];
      int r = id0 / chunks, ch = id0 - r * chunks;
#pragma unroll
      for (int q = 0; q < kPieces; ++q) {
        if (r >= MT * 32) r -= MT * 32;                    // past the end: wraps into the tile (a batch never spans it twice)
        dst[q] = r * pitch + ch * 8;
        v[q] = *reinterpret_cast<const half8*>(p.a16 + (size_t)min(r, B - 1) * K + k0 + ch * 8);
        r += step_r; ch += step_c;
        if (ch >= chunks) { ch -= chunks; r += 1; }
      }
#pragma unroll
      for (int q = 0; q < kPieces; ++q)
        if (id0 + q * NW * 64 < total) *reinterpret_cast<half8*>(sA + dst[q]) = v[q];
    };
    const int needed = (total + NW * 64 - 1) / (NW * 64);      // pieces per thread, uniform
    switch (needed < 8 ? needed : 8) {
      case 1: copy_batch(tid, std::integral_constant<int, 1>{}); break;
      case 2: copy_batch(tid, std::integral_constant<int, 2>{}); break;
      case 3: copy_batch(tid, std::integral_constant<int, 3>{}); break;
      case 4: copy_batch(tid, std::integral_constant<int, 4>{}); break;
      case 5: case 6: copy_batch(tid, std::integral_constant<int, 6>{}); break;
      default: copy_batch(tid, std::integral_constant<int, 8>{}); break;
    }
    for (int id0 = tid + NW * 64 * 8; id0 < total; id0 += NW * 64 * 4) copy_batch(id0, std::integral_constant<int, 4>{});
  }
  __syncthreads();

  // 3. MFMA over this wave's k-tiles
  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;
  const half_t* ap = sA + (lane & 31) * pitch + 8 * (lane >> 5);
  for (int base = kb; base < ke; base += kDecMaxFrag) {
#pragma unroll
    for (int u = 0; u < kDecMaxFrag; ++u) {
      if (base + u < ke) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const half8 a = *reinterpret_cast<const half8*>(ap + m * 32 * pitch + (base + u) * 16);
          acc[m] = mfma32(a, wf[u], acc[m]);
        }
      }
    }
    if (base + kDecMaxFrag < ke) {
#pragma unroll
      for (int u = 0; u < kDecMaxFrag; ++u) {
        const int kt = base + kDecMaxFrag + u;
        const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        wf[u] = (kt < ke) ? *reinterpret_cast<const half8*>(wp + (size_t)kt * 512) : z;
      }
    }
  }
  __syncthreads();          // all waves are done reading sA before it is reused

  // 4. cross-wave reduction in a fixed order
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wave * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
  __syncthreads();

  const int col = nt * 32 + (lane & 31);
  // (m, v) pairs are dealt to the waves so that every wave takes part in the epilogue
  for (int mv = wave; mv < MT * 16; mv += NW) {
    const int m = mv >> 4, v = mv & 15;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[((w * MT + m) * 16 + v) * 64 + lane];
    dec_epilogue<EPI>(p, nt, lane, m * 32 + mfma32_row(v, lane), col, s);
  }
}

// A = LayerNorm(sum_k partial_k + bias + residual), normalised in the prologue (SKIN = 0: A = the
// embedding LayerNorm of the tokens fed to the step instead, see DecGemmArgs).
// grid = ceil(column strips / NS) * ceil(B / R) workgroups, R = NW * RPW: a workgroup owns R batch rows (RPW per
// wave) of NS adjacent 32-column strips, so the redundant normalisation work per workgroup
// is R rows, not the whole batch, and it is shared by NS strips (every workgroup re-reads its rows'
// partials from L2: with one strip per workgroup that traffic is several times the weight bytes);
// the row groups of a strip read the same weight fragments (from L2 after the first).  The MFMA tile
// is fed rows 0..R-1 repeated; only the accumulator registers that hold rows < R are reduced and stored.
template <int NW, int EPI, int RC, int SKIN, int RPW, int NS = 1>
__global__ __launch_bounds__(NW * 64) void gemm_dec_ln_kernel(DecGemmArgs p) {
  constexpr int R = NW * RPW;                 // rows per workgroup: 8, 16 or 32
  constexpr int NV = R / 2;                   // accumulator registers holding rows < R (row = 8(v/4) + 4(lane/32) + v%4)
  static_assert(NW == 8 && (RPW == 1 || RPW == 2 || RPW == 4), "row groups of 8, 16 or 32 rows");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* sA = reinterpret_cast<half_t*>(smem_raw);            // [R][K + 8]
  float* red = reinterpret_cast<float*>(smem_raw);             // [NW][NS * NV][64], reused after the MFMA loop

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if ((int)blockIdx.x >= p.n_main) {      // uniform for the workgroup
    kv_prefetch_run(p.kv, blockIdx.x - p.n_main, blockIdx.x, tid, NW * 64);
    return;
  }
  const int K = p.K, B = p.B;
  const int k_tiles = K / 16;
  const int n_tiles = (p.N + 31) / 32;
  const int pitch = K + 8;
  const int kb = k_tiles * wave / NW, ke = k_tiles * (wave + 1) / NW;
  // 1-D grid of (strip groups x row groups)
  const int zg = (B + R - 1) / R;
  // XCD-contiguous order, row group fastest: the row groups of a strip group run on one XCD and share its
  // weight fragments in that L2 (measured: same speed as spreading them over XCDs, 30 % fewer HBM bytes)
  const int logical = xcd_contiguous_id(blockIdx.x, p.n_main);
  const int sg = logical / zg, zi = logical - sg * zg;
  const int row0 = zi * R;

  // strip n of this workgroup is sg * NS + n; strips past the end re-read the last one and are not stored
  const half_t* wp[NS];
  half8 wf[NS][kDecMaxFrag];
#pragma unroll
  for (int n = 0; n < NS; ++n) {
    wp[n] = p.Wp + packed_frag_offset(min(sg * NS + n, n_tiles - 1), 0, k_tiles) + lane * 8;
#pragma unroll
    for (int u = 0; u < kDecMaxFrag; ++u) {
      const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      wf[n][u] = (kb + u < ke) ? *reinterpret_cast<const half8*>(wp[n] + (size_t)(kb + u) * 512) : z;
    }
  }

  // prologue: wave w normalises rows row0 + w * RPW + i.  Loads are unconditional with clamped addresses
  // (a row >= B or a chunk past the row end re-reads a valid location and is masked): predicated loads
  // would be issued one at a time.  SKIN is a compile-time count so that the loads of every split-K
  // partial are in flight together; partials are added in index order.
  {
    const int chunks = K / 8;
    float v[RPW][RC][8], g[RC][8], bt[RC][8], bs[RC][8];
#pragma unroll
    for (int c = 0; c < RC; ++c) {
      const int cc = min(c * 64 + lane, chunks - 1);
      float4 b0 = {0.f, 0.f, 0.f, 0.f}, b1 = {0.f, 0.f, 0.f, 0.f};
      if constexpr (SKIN > 0) {
        b0 = *reinterpret_cast<const float4*>(p.bias + cc * 8);
        b1 = *reinterpret_cast<const float4*>(p.bias + cc * 8 + 4);
      }
      const float4 g0 = *reinterpret_cast<const float4*>(p.gamma + cc * 8);
      const float4 g1 = *reinterpret_cast<const float4*>(p.gamma + cc * 8 + 4);
      const float4 t0 = *reinterpret_cast<const float4*>(p.beta + cc * 8);
      const float4 t1 = *reinterpret_cast<const float4*>(p.beta + cc * 8 + 4);
      bs[c][0] = b0.x; bs[c][1] = b0.y; bs[c][2] = b0.z; bs[c][3] = b0.w;
      bs[c][4] = b1.x; bs[c][5] = b1.y; bs[c][6] = b1.z; bs[c][7] = b1.w;
      g[c][0] = g0.x; g[c][1] = g0.y; g[c][2] = g0.z; g[c][3] = g0.w;
      g[c][4] = g1.x; g[c][5] = g1.y; g[c][6] = g1.z; g[c][7] = g1.w;
      bt[c][0] = t0.x; bt[c][1] = t0.y; bt[c][2] = t0.z; bt[c][3] = t0.w;
      bt[c][4] = t1.x; bt[c][5] = t1.y; bt[c][6] = t1.z; bt[c][7] = t1.w;
    }
#pragma unroll
    for (int i = 0; i < RPW; ++i) {
      const int rr = min(row0 + wave * RPW + i, B - 1);
      if constexpr (SKIN == 0) {
        // embedding prologue: token row + position row (+ segment row); the sum is not biased
        const int fed = p.tok[rr];
        const int id = min(max(fed, 0), p.vocab_kept - 1);
        const int pos = min(p.cache_len[rr], p.max_pos - 1);
        if (p.eos >= 0 && sg == 0 && lane == 0 && row0 + wave * RPW + i < B && fed == p.eos) p.finished[rr] = 1;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
          const int cc = min(c * 64 + lane, chunks - 1);
          const half8 e = *reinterpret_cast<const half8*>(p.tok_emb + (size_t)id * K + cc * 8);
          const half8 q = *reinterpret_cast<const half8*>(p.pos_emb + (size_t)pos * K + cc * 8);
          half8 g8 = {0, 0, 0, 0, 0, 0, 0, 0};
          if (p.seg_row) g8 = *reinterpret_cast<const half8*>(p.seg_row + cc * 8);
          const float live = (c * 64 + lane < chunks) ? 1.f : 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) v[i][c][j] = ((float)e[j] + (float)q[j] + (float)g8[j]) * live;
        }
        continue;
      }
      constexpr int SKL = SKIN > 0 ? SKIN : 1;
      half8 rs[RC];
      float4 y0[SKL][RC], y1[SKL][RC];
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        const int cc = min(c * 64 + lane, chunks - 1);
        rs[c] = *reinterpret_cast<const half8*>(p.res + (size_t)rr * K + cc * 8);
#pragma unroll
        for (int s = 0; s < SKL; ++s) {
          const float* src = p.r32 + ((size_t)s * B + rr) * K + cc * 8;
          y0[s][c] = *reinterpret_cast<const float4*>(src);
          y1[s][c] = *reinterpret_cast<const float4*>(src + 4);
        }
      }
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        float a[8] = {y0[0][c].x, y0[0][c].y, y0[0][c].z, y0[0][c].w, y1[0][c].x, y1[0][c].y, y1[0][c].z, y1[0][c].w};
#pragma unroll
        for (int s = 1; s < SKL; ++s) {
          a[0] += y0[s][c].x; a[1] += y0[s][c].y; a[2] += y0[s][c].z; a[3] += y0[s][c].w;
          a[4] += y1[s][c].x; a[5] += y1[s][c].y; a[6] += y1[s][c].z; a[7] += y1[s][c].w;
        }
        const float live = (c * 64 + lane < chunks) ? 1.f : 0.f;   // the duplicated tail chunk stays out of the sums
#pragma unroll
        for (int j = 0; j < 8; ++j) v[i][c][j] = (a[j] + bs[c][j] + (float)rs[c][j]) * live;
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
      const float rs = rsqrtf(rstd[i] / (float)K + p.eps);
      const bool writer = p.xout && sg == 0 && r < B;
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        const int ch = c * 64 + lane;
        if (ch < chunks) {
          half8 o;
#pragma unroll
          for (int j = 0; j < 8; ++j) o[j] = (half_t)((v[i][c][j] - mean[i]) * rs * g[c][j] + bt[c][j]);
          *reinterpret_cast<half8*>(sA + (wave * RPW + i) * pitch + ch * 8) = o;
          if (writer) *reinterpret_cast<half8*>(p.xout + (size_t)r * K + ch * 8) = o;
        }
      }
    }
  }
  __syncthreads();

  floatx16 acc[NS];
#pragma unroll
  for (int n = 0; n < NS; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
  const half_t* ap = sA + (lane & (R - 1)) * pitch + 8 * (lane >> 5);    // tile rows R..31 repeat rows 0..R-1
  for (int base = kb; base < ke; base += kDecMaxFrag) {
#pragma unroll
    for (int u = 0; u < kDecMaxFrag; ++u)
      if (base + u < ke) {
        const half8 a = *reinterpret_cast<const half8*>(ap + (base + u) * 16);
#pragma unroll
        for (int n = 0; n < NS; ++n) acc[n] = mfma32(a, wf[n][u], acc[n]);
      }
    if (base + kDecMaxFrag < ke) {
#pragma unroll
      for (int n = 0; n < NS; ++n)
#pragma unroll
        for (int u = 0; u < kDecMaxFrag; ++u) {
          const int kt = base + kDecMaxFrag + u;
          const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
          wf[n][u] = (kt < ke) ? *reinterpret_cast<const half8*>(wp[n] + (size_t)kt * 512) : z;
        }
    }
  }
  __syncthreads();

#pragma unroll
  for (int n = 0; n < NS; ++n)
#pragma unroll
    for (int v = 0; v < NV; ++v) red[(wave * NS * NV + n * NV + v) * 64 + lane] = acc[n][v];
  __syncthreads();
  for (int nv = wave; nv < NS * NV; nv += NW) {
    const int n = nv / NV, v = nv - n * NV;
    const int nt = sg * NS + n;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[(w * NS * NV + nv) * 64 + lane];
    if (nt < n_tiles) dec_epilogue<EPI>(p, nt, lane, row0 + mfma32_row(v, lane), nt * 32 + (lane & 31), s);
  }
}

// X = LayerNorm(sum_k partial_k + bias + residual), one wave per row (launched with one row per workgroup: a row
// is 20 KB of partials at d = 1024, and four rows behind one CU's memory pipeline cost 0.4 us per launch);
// `hidden_out` optionally receives the
// fp32 widening of X.  HEAD = true is the output-head transform instead: X = LayerNorm(gelu(sum_k partial_k
// + bias)), no residual (`res` is not read).
template <int RC, bool HEAD = false>
__global__ __launch_bounds__(256) void ln_partials_kernel(const float* __restrict__ r32, int sk_in,
                                                          const float* __restrict__ bias,
                                                          const half_t* __restrict__ res, int rows, int d,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float eps,
                                                          half_t* __restrict__ X, float* __restrict__ hidden_out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);     // blockDim.x / 64 rows per workgroup
  if (r >= rows) return;
  RowRegs<RC> v;
  const int chunks = d / 8;
#pragma unroll
  for (int c = 0; c < RC; ++c) {
    const int cc = min(c * 64 + lane, chunks - 1);      // clamped: the duplicated tail chunk is never stored
    half8 rs = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (!HEAD) rs = *reinterpret_cast<const half8*>(res + (size_t)r * d + cc * 8);
    const float4 b0 = *reinterpret_cast<const float4*>(bias + cc * 8), b1 = *reinterpret_cast<const float4*>(bias + cc * 8 + 4);
    v.v[c][0] = b0.x + (float)rs[0]; v.v[c][1] = b0.y + (float)rs[1]; v.v[c][2] = b0.z + (float)rs[2];
    v.v[c][3] = b0.w + (float)rs[3]; v.v[c][4] = b1.x + (float)rs[4]; v.v[c][5] = b1.y + (float)rs[5];
    v.v[c][6] = b1.z + (float)rs[6]; v.v[c][7] = b1.w + (float)rs[7];
  }
  // partials are added in index order, up to eight buffers' loads in flight at a time (one memory round trip
  // for every split the host uses)
  constexpr int kBatch = (RC <= 2) ? 8 : 4;
  for (int s0 = 0; s0 < sk_in; s0 += kBatch) {
    float4 x0[kBatch][RC], x1[kBatch][RC];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int s = min(s0 + u, sk_in - 1);
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        const int cc = min(c * 64 + lane, chunks - 1);
        const float* src = r32 + ((size_t)s * rows + r) * d + cc * 8;
        x0[u][c] = *reinterpret_cast<const float4*>(src);
        x1[u][c] = *reinterpret_cast<const float4*>(src + 4);
      }
    }
    __builtin_amdgcn_sched_barrier(0);      // every load above is issued before the first sum below waits on one
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const float live = (s0 + u < sk_in) ? 1.f : 0.f;
#pragma unroll
      for (int c = 0; c < RC; ++c) {
        v.v[c][0] += live * x0[u][c].x; v.v[c][1] += live * x0[u][c].y; v.v[c][2] += live * x0[u][c].z;
        v.v[c][3] += live * x0[u][c].w; v.v[c][4] += live * x1[u][c].x; v.v[c][5] += live * x1[u][c].y;
        v.v[c][6] += live * x1[u][c].z; v.v[c][7] += live * x1[u][c].w;
      }
    }
  }
  if constexpr (HEAD) {
#pragma unroll
    for (int c = 0; c < RC; ++c)
#pragma unroll
      for (int j = 0; j < 8; ++j) v.v[c][j] = gelu_erf_fast(v.v[c][j]);
  }
  row_layernorm_store(v, d, lane, gamma, beta, eps, X + (size_t)r * d);
  if (hidden_out) {
    // the caller's fp32 copy is the fp16 value that feeds the projection, widened
#pragma unroll
    for (int c = 0; c < RC; ++c) {
      const int ch = c * 64 + lane;
      if (ch < chunks) {
        const half8 o = *reinterpret_cast<const half8*>(X + (size_t)r * d + ch * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) hidden_out[(size_t)r * d + ch * 8 + j] = (float)o[j];
      }
    }
  }
}

// G = gelu(sum_k partial_k + bias) as fp16 [rows, n]; one thread per 8 outputs, partial loads four at a time.
__global__ __launch_bounds__(256) void gelu_partials_kernel(const float* __restrict__ r32, int sk_in,
                                                            const float* __restrict__ bias, int rows, int n,
                                                            half_t* __restrict__ G) {
  const size_t total = (size_t)rows * n / 8;
  const size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= total) return;
  const int col = (int)((id * 8) % n);
  float a[8];
  {
    const float4 b0 = *reinterpret_cast<const float4*>(bias + col), b1 = *reinterpret_cast<const float4*>(bias + col + 4);
    a[0] = b0.x; a[1] = b0.y; a[2] = b0.z; a[3] = b0.w; a[4] = b1.x; a[5] = b1.y; a[6] = b1.z; a[7] = b1.w;
  }
  for (int s0 = 0; s0 < sk_in; s0 += 4) {
    float4 x0[4], x1[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float* src = r32 + (size_t)min(s0 + u, sk_in - 1) * rows * n + id * 8;
      x0[u] = *reinterpret_cast<const float4*>(src);
      x1[u] = *reinterpret_cast<const float4*>(src + 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float live = (s0 + u < sk_in) ? 1.f : 0.f;
      a[0] += live * x0[u].x; a[1] += live * x0[u].y; a[2] += live * x0[u].z; a[3] += live * x0[u].w;
      a[4] += live * x1[u].x; a[5] += live * x1[u].y; a[6] += live * x1[u].z; a[7] += live * x1[u].w;
    }
  }
  half8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (half_t)gelu_erf_fast(a[j]);
  *reinterpret_cast<half8*>(G + id * 8) = o;
}

}  // namespace ernie
