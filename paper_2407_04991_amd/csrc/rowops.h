// Row-wise (HBM-bound) kernels: parameter repacking, embedding gather +
// LayerNorm, bias/residual LayerNorm, last-row gather and the final argmax.
#pragma once

#include "common.h"

namespace ernie {

constexpr int kMaxRowChunks = 8;   // one wave normalises a row of up to 64 * 8 * 8 = 4096 features
// Row kernels are instantiated for RC = 2, 4, 8 chunks of 512 features per wave (d <= 1024, 2048, 4096)
// so that narrow models do not pay registers for the widest case.

// ---------------------------------------------------------------- init-time

// W [N, K] row-major fp16 -> fragment-major tiles, rows padded with zeros to a multiple of 32.
__global__ void pack_weight_kernel(const half_t* __restrict__ W, half_t* __restrict__ Wp,
                                   int N, int K, int n_tiles) {
  const int k_tiles = K / 16;
  const size_t total = (size_t)n_tiles * k_tiles * 64;
  for (size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
       id += (size_t)gridDim.x * blockDim.x) {
    const int lane = (int)(id & 63);
    const size_t frag = id >> 6;
    const int kt = (int)(frag % k_tiles);
    const int nt = (int)(frag / k_tiles);
    const int n = nt * 32 + (lane & 31);
    const int k = kt * 16 + 8 * (lane >> 5);
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (n < N) v = *reinterpret_cast<const half8*>(W + (size_t)n * K + k);
    *reinterpret_cast<half8*>(Wp + id * 8) = v;
  }
}

__global__ void cvt_f16_f32_kernel(const half_t* __restrict__ src, float* __restrict__ dst, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (float)src[i];
}

// ---------------------------------------------------------------- LayerNorm core

// One wave owns one row held as fp32 in registers: chunk c of lane l covers
// features (c * 64 + l) * 8 .. +7.  Two-pass statistics (mean, then centred
// sum of squares) in fp32, population variance, eps inside the square root.
template <int RC>
struct RowRegs {
  float v[RC][8];
};

template <int RC>
__device__ __forceinline__ void row_layernorm_store(RowRegs<RC>& r, int d, int lane, const float* __restrict__ gamma,
                                                    const float* __restrict__ beta, float eps,
                                                    half_t* __restrict__ out_row) {
  const int chunks = d / 8;
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < RC; ++c)
    if (c * 64 + lane < chunks)
#pragma unroll
      for (int j = 0; j < 8; ++j) s += r.v[c][j];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < RC; ++c)
    if (c * 64 + lane < chunks)
#pragma unroll
      for (int j = 0; j < 8; ++j) { float t = r.v[c][j] - mean; q += t * t; }
  const float rstd = rsqrtf(wave_sum(q) / (float)d + eps);
#pragma unroll
  for (int c = 0; c < RC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < chunks) {
      half8 o;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        o[j] = (half_t)((r.v[c][j] - mean) * rstd * gamma[ch * 8 + j] + beta[ch * 8 + j]);
      *reinterpret_cast<half8*>(out_row + ch * 8) = o;
    }
  }
}

// ---------------------------------------------------------------- prefill set-up

// tok_seq[t], tok_pos[t] for the packed token axis t = cu[b] + pos; also resets
// the per-sequence state: cached length = prompt length, not finished, cache row = batch row.
__global__ void token_map_kernel(const int* __restrict__ cu, int B, int T, int* __restrict__ tok_seq,
                                 int* __restrict__ tok_pos, int* __restrict__ cache_len,
                                 int* __restrict__ finished, int* __restrict__ slot) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < B) { cache_len[t] = cu[t + 1] - cu[t]; finished[t] = 0; slot[t] = t; }
  if (t >= T) return;
  int lo = 0, hi = B - 1;            // largest b with cu[b] <= t
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid - 1;
  }
  tok_seq[t] = lo;
  tok_pos[t] = t - cu[lo];
}

// x_t = LN_emb(E'[id_t] + Epos[pos_t]) for every packed prompt token (one wave per token).
template <int RC>
__global__ __launch_bounds__(256) void embed_ln_prefill_kernel(
    const int* __restrict__ ids, int Lmax, const int* __restrict__ tok_seq, const int* __restrict__ tok_pos, int T,
    const half_t* __restrict__ tok_emb, const half_t* __restrict__ pos_emb, const half_t* __restrict__ seg_row,
    const float* __restrict__ gamma, const float* __restrict__ beta, float eps, int d, half_t* __restrict__ X,
    int vocab_kept) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const int b = tok_seq[t], pos = tok_pos[t];
  const int id = min(max(ids[(size_t)b * Lmax + pos], 0), vocab_kept - 1);    // an id outside the table reads a valid row, never past it
  const half_t* e = tok_emb + (size_t)id * d;
  const half_t* p = pos_emb + (size_t)pos * d;
  RowRegs<RC> r;
  const int chunks = d / 8;
#pragma unroll
  for (int c = 0; c < RC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < chunks) {
      const half8 a = *reinterpret_cast<const half8*>(e + ch * 8);
      const half8 q = *reinterpret_cast<const half8*>(p + ch * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) r.v[c][j] = (float)a[j] + (float)q[j];
      if (seg_row) {                              // optional segment embedding: one row for the whole launch
        const half8 g = *reinterpret_cast<const half8*>(seg_row + ch * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) r.v[c][j] += (float)g[j];
      }
    }
  }
  row_layernorm_store(r, d, lane, gamma, beta, eps, X + (size_t)t * d);
}

// Decode: one token per sequence at position cache_len[b].  tok_in == NULL is
// handled by the caller passing the previous step's output buffer.
template <int RC>
__global__ __launch_bounds__(256) void embed_ln_decode_kernel(
    const int* __restrict__ tok, const int* __restrict__ cache_len, int B, int max_pos,
    const half_t* __restrict__ tok_emb, const half_t* __restrict__ pos_emb, const half_t* __restrict__ seg_row,
    const float* __restrict__ gamma, const float* __restrict__ beta, float eps, int d, half_t* __restrict__ X,
    int eos, int* __restrict__ finished, int vocab_kept) {
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);     // blockDim.x / 64 rows per workgroup
  if (b >= B) return;
  // a sequence that is fed the end-of-sequence token is finished from this step on (sticky until the next
  // prefill): later kernels of the step skip its cache and its emitted token is the end token again
  if (eos >= 0 && lane == 0 && tok[b] == eos) finished[b] = 1;
  const int pos = min(cache_len[b], max_pos - 1);
  const half_t* e = tok_emb + (size_t)min(max(tok[b], 0), vocab_kept - 1) * d;
  const half_t* p = pos_emb + (size_t)pos * d;
  RowRegs<RC> r;
  const int chunks = d / 8;
#pragma unroll
  for (int c = 0; c < RC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < chunks) {
      const half8 a = *reinterpret_cast<const half8*>(e + ch * 8);
      const half8 q = *reinterpret_cast<const half8*>(p + ch * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) r.v[c][j] = (float)a[j] + (float)q[j];
      if (seg_row) {                              // optional segment embedding: one row for the whole launch
        const half8 g = *reinterpret_cast<const half8*>(seg_row + ch * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) r.v[c][j] += (float)g[j];
      }
    }
  }
  row_layernorm_store(r, d, lane, gamma, beta, eps, X + (size_t)b * d);
}

// X = LN(Y) where Y already holds sublayer output + bias + residual (fp16 rows, prefill).
template <int RC>
__global__ __launch_bounds__(256) void ln_rows_f16_kernel(const half_t* __restrict__ Y, int rows, int d,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float eps,
                                                          half_t* __restrict__ X) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= rows) return;
  RowRegs<RC> r;
  const int chunks = d / 8;
#pragma unroll
  for (int c = 0; c < RC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < chunks) {
      const half8 a = *reinterpret_cast<const half8*>(Y + (size_t)t * d + ch * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) r.v[c][j] = (float)a[j];
    }
  }
  row_layernorm_store(r, d, lane, gamma, beta, eps, X + (size_t)t * d);
}

// Last valid prompt row of every sequence -> dense [B, d] (fp16 for the logits
// GEMM, optional fp32 copy for the caller).
__global__ void gather_last_rows_kernel(const half_t* __restrict__ X, const int* __restrict__ cu, int B, int d,
                                        half_t* __restrict__ Hlast, float* __restrict__ hidden_out) {
  const int b = blockIdx.x;
  const half_t* src = X + (size_t)(cu[b + 1] - 1) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const half_t v = src[i];
    Hlast[(size_t)b * d + i] = v;
    if (hidden_out) hidden_out[(size_t)b * d + i] = (float)v;
  }
}

// Second argmax stage: one block per sequence reduces the per-strip candidates
// (value, index); the lowest index wins exact ties.  Also advances the cached
// length of the sequence after a decode step (advance = 1).  A finished sequence
// (`finished` non-null and set) emits `eos` and does not advance.  `step_counter` (may be null) is advanced by
// one: the number of the decode step that tags the hand-overs of the one-launch decode kernel.
__global__ __launch_bounds__(256) void argmax_final_kernel(const float* __restrict__ strip_val,
                                                           const int* __restrict__ strip_idx, int strips,
                                                           int* __restrict__ tok_out, int* __restrict__ tok_keep,
                                                           int* __restrict__ cache_len, int advance, int max_seq, int vocab,
                                                           const int* __restrict__ finished, int eos,
                                                           unsigned* __restrict__ step_counter = nullptr) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int b = blockIdx.x;
  if (step_counter && b == 0 && threadIdx.x == 0) *step_counter += 1u;
  // everything this workgroup reads is requested up front: the row's state for the last step of thread 0 and
  // the first four candidates of every thread (a loop of load + compare costs a memory round trip per trip)
  int done_flag = 0, len_now = 0;
  if (threadIdx.x == 0) {
    done_flag = finished ? finished[b] : 0;
    len_now = advance ? cache_len[b] : 0;
  }
  float v = -INFINITY;
  int i = 0x7fffffff;
  {
    float cv[4];
    int ci[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int s = min((int)threadIdx.x + q * 256, strips - 1);       // clamped: a duplicate candidate changes nothing
      cv[q] = strip_val[(size_t)b * strips + s];
      ci[q] = strip_idx[(size_t)b * strips + s];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) argmax_merge(v, i, cv[q], ci[q]);
  }
  for (int s = threadIdx.x + 4 * 256; s < strips; s += blockDim.x)
    argmax_merge(v, i, strip_val[(size_t)b * strips + s], strip_idx[(size_t)b * strips + s]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(v, o, 64);
    const int oi = __shfl_xor(i, o, 64);
    argmax_merge(v, i, ov, oi);
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = v; si[threadIdx.x >> 6] = i; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) argmax_merge(v, i, sv[w], si[w]);
    if (i < 0 || i >= vocab) i = 0;   // only reachable if every logit is NaN
    const bool done = done_flag != 0;
    if (done) i = eos;
    tok_out[b] = i;
    if (tok_keep != tok_out) tok_keep[b] = i;
    if (advance && !done && len_now < max_seq) cache_len[b] = len_now + 1;
  }
}

// Batch compaction: row i of the per-sequence state takes the values of row keep[i] (keep ascending,
// n_keep <= 256).  One workgroup: every thread reads its source row before anyone writes.
__global__ __launch_bounds__(256) void batch_compact_kernel(const int* __restrict__ keep, int n_keep,
                                                            int* __restrict__ cache_len, int* __restrict__ tok_prev,
                                                            int* __restrict__ finished, int* __restrict__ slot) {
  const int t = threadIdx.x;
  int a = 0, b = 0, c = 0, e = 0;
  if (t < n_keep) {
    const int src = keep[t];
    a = cache_len[src]; b = tok_prev[src]; c = finished[src]; e = slot[src];
  }
  __syncthreads();
  if (t < n_keep) { cache_len[t] = a; tok_prev[t] = b; finished[t] = c; slot[t] = e; }
}

__global__ __launch_bounds__(256) void copy_ints_kernel(const int* __restrict__ src, int* __restrict__ dst, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

}  // namespace ernie
