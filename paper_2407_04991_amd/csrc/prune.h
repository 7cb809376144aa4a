// Vocabulary trimming kernels (paper: Method, "Embedding layer pruning"):
// frequency count, exact top-k selection with reserved ids, id maps, row gather.
// All integer work; every result is exact and independent of scheduling.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ernie {

typedef unsigned long long u64_t;

constexpr int kCountThreads = 1024;
constexpr int kCountMaxLdsVocab = 36864;   // 144 KiB of 32-bit bins

// Occurrence count.  Each workgroup owns a private 32-bit histogram in LDS (a
// workgroup sees fewer than 2^32 tokens: the host bounds n and gridDim.x) and
// adds its non-zero bins to the 64-bit totals at the end, so global atomics are
// V per workgroup instead of one per token.  LDS = false counts straight into
// the totals (vocabularies too large for LDS).
// The stream is read as 16-byte vectors from the first aligned element on;
// the unaligned head and the tail (< 4 elements each) go to workgroup 0.
template <bool LDS>
__global__ __launch_bounds__(kCountThreads) void vocab_count_kernel(const int* __restrict__ ids, long long n, int V,
                                                                    u64_t* __restrict__ counts) {
  extern __shared__ unsigned int hist[];
  const int tid = threadIdx.x;
  if constexpr (LDS) {
    for (int i = tid; i < V; i += kCountThreads) hist[i] = 0;
    __syncthreads();
  }
  auto add = [&](int t) {
    if ((unsigned)t < (unsigned)V) {
      if constexpr (LDS) atomicAdd(&hist[t], 1u);
      else atomicAdd(&counts[t], (u64_t)1);
    }
  };
  const long long head = min(n, (long long)(((16 - ((uintptr_t)ids & 15)) & 15) / 4));
  const long long nvec = (n - head) / 4;
  const int4* v = reinterpret_cast<const int4*>(ids + head);
  const long long stride = (long long)gridDim.x * kCountThreads;
  long long i = (long long)blockIdx.x * kCountThreads + tid;
  for (; i + 3 * stride < nvec; i += 4 * stride) {          // four loads in flight per lane
    const int4 a = v[i], b = v[i + stride], c = v[i + 2 * stride], e = v[i + 3 * stride];
    add(a.x); add(a.y); add(a.z); add(a.w);
    add(b.x); add(b.y); add(b.z); add(b.w);
    add(c.x); add(c.y); add(c.z); add(c.w);
    add(e.x); add(e.y); add(e.z); add(e.w);
  }
  for (; i < nvec; i += stride) {
    const int4 a = v[i];
    add(a.x); add(a.y); add(a.z); add(a.w);
  }
  if (blockIdx.x == 0) {
    const long long tail0 = head + 4 * nvec;
    if (tid < head) add(ids[tid]);
    if (tail0 + tid < n) add(ids[tail0 + tid]);             // n - tail0 < 4
  }
  if constexpr (LDS) {
    __syncthreads();
    for (int j = tid; j < V; j += kCountThreads) {
      const unsigned int c = hist[j];
      if (c) atomicAdd(&counts[j], (u64_t)c);
    }
  }
}

struct ReservedIds {
  int n;
  int id[16];
};

// Selection by exact rank: id i is kept iff fewer than k ids are preferred to it.
// Preference is the strict total order (reserved, count, lower id), so exactly k
// ids pass.  One thread per id; the keys of all ids stream through LDS in tiles
// (every lane reads the same LDS word: a broadcast, no bank conflicts).
constexpr int kRankThreads = 256, kRankTile = 1024;

__device__ __forceinline__ u64_t select_key(const u64_t* __restrict__ counts, int j, const ReservedIds& res) {
  bool f = false;
#pragma unroll
  for (int r = 0; r < 16; ++r) f |= (r < res.n) && (res.id[r] == j);
  return (counts[j] & 0x7FFFFFFFFFFFFFFFull) | ((u64_t)f << 63);
}

__global__ __launch_bounds__(256) void fill_int_kernel(int* __restrict__ p, int n, int v) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// gridDim.y slices of the id range are compared by different workgroups; the partial counts are added
// into rank[i] (zeroed beforehand), integers, so the sum does not depend on the order.
__global__ __launch_bounds__(kRankThreads) void vocab_rank_kernel(const u64_t* __restrict__ counts, int V,
                                                                  ReservedIds res, int* __restrict__ rank_out) {
  __shared__ u64_t tile[kRankTile];
  const int tid = threadIdx.x;
  const int i = blockIdx.x * kRankThreads + tid;
  const u64_t ki = (i < V) ? select_key(counts, i, res) : 0;
  const int tiles = (V + kRankTile - 1) / kRankTile;
  const int t_beg = (int)((long long)tiles * blockIdx.y / gridDim.y), t_end = (int)((long long)tiles * (blockIdx.y + 1) / gridDim.y);
  int rank = 0;
  for (int tt = t_beg; tt < t_end; ++tt) {
    const int j0 = tt * kRankTile;
    __syncthreads();
    for (int t = tid; t < kRankTile; t += kRankThreads) tile[t] = (j0 + t < V) ? select_key(counts, j0 + t, res) : 0;
    __syncthreads();
    const int lim = min(kRankTile, V - j0);
    for (int t = 0; t < lim; ++t) {
      const u64_t kj = tile[t];
      rank += (kj > ki) || (kj == ki && (j0 + t) < i);
    }
  }
  if (i < V && rank) atomicAdd(&rank_out[i], rank);
}

// Compaction by one workgroup: `map` holds the ranks on entry (id i is kept iff rank < k); on exit
// map[i] = trimmed index of full id i (dropped ids: the trimmed index of `unk`)
// and kept_ids[t] = full id of trimmed index t, ascending.
constexpr int kCompactThreads = 1024;

__global__ __launch_bounds__(kCompactThreads) void vocab_compact_kernel(int* __restrict__ map, int V, int k, int unk,
                                                                        int* __restrict__ kept_ids) {
  __shared__ int wsum[kCompactThreads / 64];
  __shared__ int s_base, s_unk;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { s_base = 0; s_unk = 0; }
  __syncthreads();
  for (int c0 = 0; c0 < V; c0 += kCompactThreads) {
    const int i = c0 + tid;
    const int f = (i < V && map[i] < k) ? 1 : 0;
    int x = f;                                              // inclusive scan inside the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(x, o, 64);
      if (lane >= o) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    int woff = 0;
    for (int w = 0; w < wave; ++w) woff += wsum[w];
    const int base = s_base;
    const int excl = base + woff + x - f;
    if (i < V) {
      if (f) {
        kept_ids[excl] = i;
        map[i] = excl;
        if (i == unk) s_unk = excl;
      } else {
        map[i] = -1;
      }
    }
    __syncthreads();                                        // s_base and wsum have been read by everyone
    if (tid == kCompactThreads - 1) s_base = base + woff + x;
    __syncthreads();
  }
  const int u = s_unk;
  for (int i = tid; i < V; i += kCompactThreads)
    if (map[i] < 0) map[i] = u;                             // the same thread wrote map[i] above
}

// table_kept[i, :] = table_full[kept_ids[i], :] in 16-byte pieces (d8 = d / 8 pieces per row).
__global__ __launch_bounds__(256) void vocab_gather_rows_kernel(const int4* __restrict__ full, int V, int d8,
                                                                const int* __restrict__ kept_ids, int k,
                                                                int4* __restrict__ out) {
  const long long total = (long long)k * d8;
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const int row = (int)(idx / d8), c = (int)(idx - (long long)row * d8);
    const int src = min(max(kept_ids[row], 0), V - 1);
    out[idx] = full[(long long)src * d8 + c];
  }
}

// out[i] = map[in[i]] inside the table, fallback outside; 16-byte vectors when both streams are aligned alike.
__global__ __launch_bounds__(256) void remap_ids_kernel(const int* in, long long n, const int* __restrict__ map,
                                                        int map_len, int fallback, int* out, int vec_ok) {
  auto look = [&](int t) { return ((unsigned)t < (unsigned)map_len) ? map[t] : fallback; };
  const long long stride = (long long)gridDim.x * 256;
  const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
  if (vec_ok) {
    const long long nvec = n / 4;
    const int4* vi = reinterpret_cast<const int4*>(in);
    int4* vo = reinterpret_cast<int4*>(out);
    long long i = g;
    for (; i + 3 * stride < nvec; i += 4 * stride) {       // four vectors (16 table lookups) in flight per lane
      const int4 a = vi[i], b = vi[i + stride], c = vi[i + 2 * stride], e = vi[i + 3 * stride];
      const int4 ra = int4{look(a.x), look(a.y), look(a.z), look(a.w)};
      const int4 rb = int4{look(b.x), look(b.y), look(b.z), look(b.w)};
      const int4 rc = int4{look(c.x), look(c.y), look(c.z), look(c.w)};
      const int4 re = int4{look(e.x), look(e.y), look(e.z), look(e.w)};
      vo[i] = ra; vo[i + stride] = rb; vo[i + 2 * stride] = rc; vo[i + 3 * stride] = re;
    }
    for (; i < nvec; i += stride) {
      const int4 a = vi[i];
      vo[i] = int4{look(a.x), look(a.y), look(a.z), look(a.w)};
    }
    for (long long i = 4 * nvec + g; i < n; i += stride) out[i] = look(in[i]);
  } else {
    for (long long i = g; i < n; i += stride) out[i] = look(in[i]);
  }
}

}  // namespace ernie
