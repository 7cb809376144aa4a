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
constexpr float kLog2e = 1.44269504088896340736f;
constexpr int kAttnTile = kAttnKBlock * 128;      // bytes of one staged tile: 64 cache rows (keys) x 128 bytes (head dim)
constexpr int kAttnLdsBytes = 4 * kAttnTile;      // K and V tiles, double-buffered

typedef __attribute__((address_space(1))) const void attn_global_cptr_t;
typedef __attribute__((address_space(3))) void attn_lds_ptr_t;
typedef short attn_short4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) attn_short4 attn_lds_short4_t;

// The K and V rows of a key block are copied once per workgroup, global -> LDS directly, 64 rows x 128 bytes
// each, one block ahead of the arithmetic.  16-byte chunk c of row r sits in slot
//   K tile:  c ^ ((r / 2) % 8)      the 16 lanes served together by a 16-byte read (16 rows, one logical chunk)
//                                   touch 64 distinct banks
//   V tile:  c ^ (4 * ((r / 2) % 2))  the 32 lanes served together by an 8-byte transposing read (4 rows x 64
//                                   bytes) touch 64 distinct banks
//
// Scores are produced transposed (S^T = K Q^T) so that every lane owns ONE query column: softmax statistics
// are per-lane plus one exchange with lane^32, and the probabilities, still in registers, are directly the
// B operand of O^T = V^T P^T: accumulator registers 8 c .. 8 c + 7 of lane half hh hold keys
// 16 c + 4 hh + {0..3} and 16 c + 8 + 4 hh + {0..3} of a 32-key tile.  The matching A operand (8 keys of one
// head-dim index per lane) comes out of the row-major V tile through the LDS transposing read
// (ds_read_b64_tr_b16): in every group of 16 lanes, lane s supplies the address of 4 consecutive 16-bit
// elements and lane i receives element i % 4 of the chunks of lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.
// With lane s pointing at key (s / 4), head-dim elements 4 (s % 4) .. + 3 of a 4-key x 16-element patch, lane i
// receives the patch's 4 keys at element i: two such reads make one fragment.
// (min 2 waves per SIMD: with a register budget of 256 the compiler keeps the MFMA accumulators in
// ordinary registers instead of shuttling them through the accumulation file around every block.)
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(const half_t* __restrict__ Q,      // [H][T][64]
                                                              const half_t* __restrict__ Kc,     // layer K cache
                                                              const half_t* __restrict__ Vc,     // layer V cache
                                                              const int* __restrict__ cu, int T, int H, int S, int d,
                                                              half_t* __restrict__ O) {           // [T, d]
  // Dynamic LDS (kAttnLdsBytes): for a statically declared array the compiler makes every LDS read wait for all
  // outstanding direct-to-LDS copies, the ones just issued for the other buffer included.
  extern __shared__ __align__(16) unsigned char smem_attn[];
  unsigned char (*sK)[kAttnTile] = reinterpret_cast<unsigned char (*)[kAttnTile]>(smem_attn);
  unsigned char (*sV)[kAttnTile] = reinterpret_cast<unsigned char (*)[kAttnTile]>(smem_attn + 2 * kAttnTile);

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

  // copies: a wave instruction moves 8 whole rows (lane -> row lane / 8, slot lane % 8); every thread issues two
  // per tile.  Rows past the end of the sequence re-read its last key (valid memory): their scores are masked,
  // so their (finite) values only ever meet a zero probability.
  int st_row[2], st_k[2], st_v[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int id = tid + 256 * i;
    st_row[i] = id >> 3;
    st_k[i] = ((id & 7) ^ ((st_row[i] >> 1) & 7)) * 8;            // halves: the global chunk that lands in slot id % 8
    st_v[i] = ((id & 7) ^ (((st_row[i] >> 1) & 1) << 2)) * 8;
  }
  auto fetch_block = [&](int kb0, int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const size_t key = (size_t)min(kb0 + st_row[i], L - 1) * 64;
      const int dst = (wave * 8 + 32 * i) * 128;
      __builtin_amdgcn_global_load_lds((attn_global_cptr_t*)(Kb + key + st_k[i]), (attn_lds_ptr_t*)(sK[buf] + dst), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((attn_global_cptr_t*)(Vb + key + st_v[i]), (attn_lds_ptr_t*)(sV[buf] + dst), 16, 0, 0);
    }
  };
  fetch_block(0, 0);

  // K fragment reads: tile row 32 kk + lane % 32, logical chunk 2 c + hh
  const int r = lane & 31;
  int k_off[2], k_swz[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) { k_off[x] = (32 * x + r) * 128; k_swz[x] = ((32 * x + r) >> 1) & 7; }
  // V transposing reads: as a source, this lane points at key 4 hh + (lane % 16) / 4 of an 8-key group and at
  // head-dim elements 16 ((lane / 16) % 2) + 4 (lane % 4) .. + 3 of the 32-element tile half m
  const int l16 = lane & 15;
  const int v_row = 4 * hh + (l16 >> 2);                               // + 16 c + 8 t
  const int v_chunk = 2 * ((lane >> 4) & 1) + ((l16 >> 1) & 1);        // + 4 m, then ^ 4 * ((row / 2) % 2)
  const int v_base = v_row * 128 + 8 * (l16 & 1);
  const int v_flip = ((v_row >> 1) & 1) << 2;

  floatx16 o[2];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[m][v] = 0.f;
  float row_max = -INFINITY, row_sum = 0.f;     // row_max is kept pre-multiplied by log2(e)

  int buf = 0;
  for (int kb0 = 0; kb0 < L; kb0 += kAttnKBlock, buf ^= 1) {
    __syncthreads();            // waits for this wave's copies of the block, then for everybody's
    // the other buffer pair was last read before that barrier: refill it during this block's arithmetic
    if (kb0 + kAttnKBlock < L) fetch_block(kb0 + kAttnKBlock, buf ^ 1);

    // S^T[key][query] for the 64 keys of the block x this wave's 32 queries (two 32-key MFMA tiles), then ONE
    // online-softmax update for the whole block
    floatx16 sc[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sc[kk][v] = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const half8 kf = *reinterpret_cast<const half8*>(sK[buf] + k_off[kk] + (((2 * c + hh) ^ k_swz[kk]) * 16));
        sc[kk] = mfma32(kf, qf[c], sc[kk]);
      }
    }
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
    // exp(s - max) = exp2(s * log2(e) - max2): one multiply-add and one exponential per score
    const float m_new = fmaxf(row_max, mx * kLog2e);     // finite: the block holds at least one valid key
    if (__any(m_new > row_max)) {                        // the running maximum rarely moves after the first blocks
      const float alpha = exp2f(row_max - m_new);        // exp2(-inf) = 0 on the first block
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
        const float p = __builtin_amdgcn_exp2f(fmaf(sc[kk][v], kLog2e, -row_max));
        ps += p;
        pf[2 * kk + (v >> 3)][v & 7] = (half_t)p;
      }
    ps += __shfl_xor(ps, 32, 64);
    row_sum += ps;
    // O^T[e][query] += V^T[e][keys] * P^T[keys][query]; MFMA step c covers keys 16 c .. 16 c + 15 of the block
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        half4 part[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
          part[t] = __builtin_bit_cast(half4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((attn_lds_short4_t*)(
              sV[buf] + v_base + (16 * c + 8 * t) * 128 + (((4 * m + v_chunk) ^ v_flip) * 16))));
        const half8 vf = {part[0][0], part[0][1], part[0][2], part[0][3], part[1][0], part[1][1], part[1][2], part[1][3]};
        o[m] = mfma32(vf, pf[c], o[m]);
      }
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
                                                                    const int* __restrict__ slot,       // cache row of batch row b; null = b
                                                                    DecPrefetch warm) {                 // grid rows >= B only warm the L2 (small vectors)
  __shared__ float sm[NW][8][10];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int h = blockIdx.x, b = blockIdx.y;
  if (b >= B) {      // uniform for the workgroup
    dec_prefetch_run(warm, h + H * (b - B), h + H * b, tid, NW * 64);
    return;
  }
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
