// Attention kernels over the head-major key/value cache
// [Bmax][H][S][64] fp16 (each (sequence, head) stream is contiguous).
//
//  - attn_prefill_kernel: bidirectional attention of every prompt query over
//    the valid prompt keys of its own sequence (padding never stored nor seen),
//    flash-style on MFMA with fp32 online softmax.
//  - attn_decode_fused_kernel: one query per (sequence, head) over all cached keys,
//    a pure streaming read of K and V with wave-shuffle softmax reductions; the
//    new token's q, k, v come from the raw QKV GEMM output (+ bias) in its prologue.
#pragma once

#include "common.h"

namespace ernie {

// ---------------------------------------------------------------- prefill

constexpr int kAttnQTile = 128;            // queries per workgroup (32 per wave)
constexpr int kAttnKBlock = 64;            // keys staged per iteration
constexpr int kAttnVtPitch = kAttnKBlock + 4;   // halves; 136-byte pitch spreads 8-byte reads over all banks

// Scores are produced transposed (S^T = K Q^T) so that every lane owns ONE
// query column: softmax statistics are per-lane plus one exchange with lane^32.
// The probabilities, still in registers, are directly the B operand of
// O^T = V^T P^T provided V^T is read with the matching key permutation
// (slot (half, j) of k-step c  <->  key 16c + 8(j/4) + 4*half + j%4).
__global__ __launch_bounds__(256) void attn_prefill_kernel(const half_t* __restrict__ Q,      // [H][T][64]
                                                           const half_t* __restrict__ Kc,     // layer K cache
                                                           const half_t* __restrict__ Vc,     // layer V cache
                                                           const int* __restrict__ cu, int T, int H, int S, int d,
                                                           half_t* __restrict__ O) {           // [T, d]
  __shared__ __align__(16) half_t sVt[64 * kAttnVtPitch];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int h = blockIdx.y, b = blockIdx.z;
  const int t0 = cu[b];
  const int L = cu[b + 1] - t0;
  const int qbase = blockIdx.x * kAttnQTile;
  if (qbase >= L) return;                       // uniform for the whole workgroup

  const int hh = lane >> 5;
  const int qi = qbase + wave * 32 + (lane & 31);    // this lane's query
  const bool q_ok = qi < L;

  // Q fragments (B operand, k = head-dim index), pre-scaled by 1/sqrt(64) (exact in fp16)
  half8 qf[4];
  {
    const half_t* qp = Q + ((size_t)h * T + t0 + (q_ok ? qi : 0)) * 64 + 8 * hh;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (q_ok) v = *reinterpret_cast<const half8*>(qp + 16 * c);
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = v[j] * (half_t)0.125f;
      qf[c] = v;
    }
  }

  const half_t* Kb = Kc + ((size_t)b * H + h) * S * 64;
  const half_t* Vb = Vc + ((size_t)b * H + h) * S * 64;

  floatx16 o[2];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[m][v] = 0.f;
  float row_max = -INFINITY, row_sum = 0.f;

  // Operands of a key block are fetched one block ahead: V rows (two 16-byte pieces per thread, transposed into
  // LDS at the top of the block's iteration) and this wave's K fragments.  Rows past the end of the sequence
  // re-read its last key (always valid memory); they are masked / zeroed where it matters.
  half8 vreg[2], kf[2][4];
  auto fetch_block = [&](int kb0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i;
      const int key = min(kb0 + (id >> 3), L - 1), ec = id & 7;
      vreg[i] = *reinterpret_cast<const half8*>(Vb + (size_t)key * 64 + ec * 8);
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int krow = min(kb0 + kk * 32 + (lane & 31), L - 1);
#pragma unroll
      for (int c = 0; c < 4; ++c) kf[kk][c] = *reinterpret_cast<const half8*>(Kb + (size_t)krow * 64 + 16 * c + 8 * hh);
    }
  };
  fetch_block(0);

  for (int kb0 = 0; kb0 < L; kb0 += kAttnKBlock) {
    // stage V^T of this key block: thread handles key = id / 8, 8 head-dim values at (id % 8) * 8
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i;
      const int key = id >> 3, ec = id & 7;
      const bool live = kb0 + key < L;                      // keys past the end contribute V = 0
#pragma unroll
      for (int j = 0; j < 8; ++j) sVt[(ec * 8 + j) * kAttnVtPitch + key] = live ? vreg[i][j] : (half_t)0.f;
    }
    __syncthreads();

    // S^T[key][query] for the 64 keys of the block x this wave's 32 queries (two 32-key MFMA tiles), then ONE
    // online-softmax update for the whole block
    floatx16 sc[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sc[kk][v] = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) sc[kk] = mfma32(kf[kk][c], qf[c], sc[kk]);
    }
    if (kb0 + kAttnKBlock < L) fetch_block(kb0 + kAttnKBlock);      // next block's loads fly during softmax and P V
    if (kb0 + kAttnKBlock > L) {                   // only the last block of a sequence has keys to mask (uniform branch)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kb0 + kk * 32 + mfma32_row(v, lane) >= L) sc[kk][v] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sc[kk][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(row_max, mx);              // finite: the block holds at least one valid key
    if (__any(m_new > row_max)) {                        // the running maximum rarely moves after the first blocks
      const float alpha = __expf(row_max - m_new);       // exp(-inf) = 0 on the first block
      row_sum *= alpha;
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[m][v] *= alpha;
      row_max = m_new;
    }
    float ps = 0.f;
    half8 pf[4];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __expf(sc[kk][v] - row_max);
        ps += p;
        pf[2 * kk + (v >> 3)][v & 7] = (half_t)p;
      }
    ps += __shfl_xor(ps, 32, 64);
    row_sum += ps;
    // O^T[e][query] += V^T[e][keys] * P^T[keys][query]
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const half_t* vt = sVt + (32 * m + (lane & 31)) * kAttnVtPitch + 4 * hh;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const half4 lo = *reinterpret_cast<const half4*>(vt + 16 * c);
        const half4 hi = *reinterpret_cast<const half4*>(vt + 16 * c + 8);
        half8 vf;
        vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
        vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
        o[m] = mfma32(vf, pf[c], o[m]);
      }
    }
    __syncthreads();
  }

  if (q_ok) {
    const float inv = 1.0f / row_sum;
    half_t* op = O + (size_t)(t0 + qi) * d + h * 64;
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        half4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (half_t)(o[m][4 * g + j] * inv);
        *reinterpret_cast<half4*>(op + 32 * m + 8 * g + 4 * hh) = w;
      }
  }
}

// ---------------------------------------------------------------- decode

// One workgroup (NW waves) per (head, sequence).  Lane l of a wave reads 16
// bytes (8 head-dim values, chunk l % 8) of key row (l / 8) of an 8-row group,
// so one wave load instruction covers 1 KiB of contiguous cache.  Wave w takes
// U consecutive 8-row groups out of every NW * U.  Every 8-lane team keeps an online
// softmax (max, sum, 8 output values) over its own rows; teams are merged by
// shuffles, waves through LDS.
struct SoftmaxPart {
  float m, l, acc[8];
};

__device__ __forceinline__ void softmax_merge(SoftmaxPart& a, float om, float ol, const float* oacc) {
  const float mn = fmaxf(a.m, om);
  const float sa = (a.m == -INFINITY) ? 0.f : __expf(a.m - mn);
  const float sb = (om == -INFINITY) ? 0.f : __expf(om - mn);
  a.l = a.l * sa + ol * sb;
#pragma unroll
  for (int j = 0; j < 8; ++j) a.acc[j] = a.acc[j] * sa + oacc[j] * sb;
  a.m = mn;
}

// The QKV epilogue is folded into the prologue:
// q, k, v of the new token are raw fp32 GEMM outputs [B, 3d] (split-K partials) plus bias; the
// new key and value are rounded to fp16, appended to the cache (slot
// cache_len[b]) and used from registers, so the cache is never read back in
// the kernel that writes it.
//
// NW waves, U groups in flight per wave: one batch covers NW * U * 8 keys, and the host picks
// (NW, U) so that a short cache is covered by a single batch.  The first batch is requested before
// the cached length is known (bounded by the capacity S only: the cache is allocated up to S, and
// whatever lies past the valid length is masked out after the fact), so the length, the cache
// stream and the raw q, k, v are all fetched in one memory round trip instead of three.
template <bool NT>
__device__ __forceinline__ half8 load_kv(const half_t* p) {
  // NT: streaming hint -- the cache rows are read once per step and should not displace the weights
  // from the caches in front of HBM
  if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const half8*>(p));
  else return *reinterpret_cast<const half8*>(p);
}

template <int NW, int U, bool NT = false>
__global__ __launch_bounds__(NW * 64) void attn_decode_fused_kernel(const float* __restrict__ Rqkv,   // [sk_in][B, 3d] fp32 split-K partials
                                                                    int sk_in, int B,
                                                                    const float* __restrict__ bqkv,   // [3d]
                                                                    half_t* __restrict__ Kc, half_t* __restrict__ Vc,
                                                                    const int* __restrict__ cache_len, int H, int S,
                                                                    int d, half_t* __restrict__ O,
                                                                    const int* __restrict__ finished,   // [B] or null (no end-of-sequence id set)
                                                                    const int* __restrict__ slot) {     // cache row of batch row b; null = b
  __shared__ float sm[NW][8][10];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int h = blockIdx.x, b = blockIdx.y;
  const int ec = lane & 7, team = lane >> 3;
  if (finished && finished[b]) return;           // finished sequence: no cache stream, no append; its output row is not used
  const int cb = slot ? slot[b] : b;             // after a batch compaction the cache rows are no longer the batch rows
  half_t* Kb = Kc + ((size_t)cb * H + h) * S * 64 + ec * 8;
  half_t* Vb = Vc + ((size_t)cb * H + h) * S * 64 + ec * 8;

  half8 kf[U], vf[U];
  int key[U];
  int g0 = wave * U;
  // first batch: addresses clamped to the capacity, validity decided later
#pragma unroll
  for (int u = 0; u < U; ++u) {
    key[u] = (g0 + u) * 8 + team;
    const size_t row = (size_t)min(key[u], S - 1) * 64;
    kf[u] = load_kv<NT>(Kb + row);
    vf[u] = load_kv<NT>(Vb + row);
  }
  const int len = cache_len[b];

  float q[8];
  half8 knew, vnew;
  {
    const float* r = Rqkv + (size_t)b * 3 * d + h * 64 + ec * 8;
    const float* bs = bqkv + h * 64 + ec * 8;
    float aq[8], ak[8], av[8];
    if (sk_in == 1) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { aq[j] = r[j] + bs[j]; ak[j] = r[d + j] + bs[d + j]; av[j] = r[2 * d + j] + bs[2 * d + j]; }
    } else {
      // split-K partials (at most 8): team t fetches partial t, so all of them arrive in one memory round
      // trip; the teams are then summed by a fixed butterfly (same order on every run)
      const float live = (team < sk_in) ? 1.f : 0.f;
      const float* rs = r + (size_t)min(team, sk_in - 1) * B * 3 * d;
#pragma unroll
      for (int j = 0; j < 8; ++j) { aq[j] = rs[j] * live; ak[j] = rs[d + j] * live; av[j] = rs[2 * d + j] * live; }
#pragma unroll
      for (int off = 8; off < 64; off <<= 1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          aq[j] += __shfl_xor(aq[j], off, 64); ak[j] += __shfl_xor(ak[j], off, 64); av[j] += __shfl_xor(av[j], off, 64);
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) { aq[j] += bs[j]; ak[j] += bs[d + j]; av[j] += bs[2 * d + j]; }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      q[j] = (float)(half_t)aq[j] * 0.125f;                 // q passes through fp16 like every stored activation
      knew[j] = (half_t)ak[j];
      vnew[j] = (half_t)av[j];
    }
  }
  const bool has_new = len < S;                 // a replayed step past capacity appends nothing
  const int c = has_new ? len + 1 : S;
  const int newest = has_new ? len : -1;        // this key comes from registers, not from the cache
  if (has_new && wave == 0 && team == 0) {
    *reinterpret_cast<half8*>(Kb + (size_t)len * 64) = knew;
    *reinterpret_cast<half8*>(Vb + (size_t)len * 64) = vnew;
  }

  SoftmaxPart st;
  st.m = -INFINITY; st.l = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] = 0.f;

  while (g0 * 8 < c) {
    float s[U];
    float mx = st.m;
    half8 vcur[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool valid = key[u] < c;
      const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      if (key[u] == newest) { kf[u] = knew; vf[u] = vnew; }
      float p = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) p += q[j] * (float)kf[u][j];
      p += __shfl_xor(p, 1, 64);
      p += __shfl_xor(p, 2, 64);
      p += __shfl_xor(p, 4, 64);
      s[u] = valid ? p : -INFINITY;
      vcur[u] = valid ? vf[u] : z;               // rows past the valid length hold arbitrary bits: weight 0 must meet value 0
      mx = fmaxf(mx, s[u]);
    }
    g0 += NW * U;
    if (g0 * 8 < c) {                            // next batch in flight during the softmax update
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
        const float p = __expf(s[u] - mx);
        st.l += p;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[j] += p * (float)vcur[u][j];
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
    sm[wave][ec][0] = st.m; sm[wave][ec][1] = st.l;
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[wave][ec][2 + j] = st.acc[j];
  }
  __syncthreads();
  if (wave == 0 && team == 0) {
#pragma unroll
    for (int w = 1; w < NW; ++w) softmax_merge(st, sm[w][ec][0], sm[w][ec][1], &sm[w][ec][2]);
    const float inv = 1.0f / st.l;
    half8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (half_t)(st.acc[j] * inv);
    *reinterpret_cast<half8*>(O + (size_t)b * d + h * 64 + ec * 8) = o;
  }
}

}  // namespace ernie
