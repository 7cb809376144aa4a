// C ABI of the vocabulary-trimming step (see include/ernie_prune.h): host-side
// argument checks and kernel launches.  Nothing here allocates device memory.

#include "../../include/ernie.h"
#include "../../include/ernie_prune.h"

#include <hip/hip_runtime.h>

#include <algorithm>

#include "prune.h"

using namespace ernie;

namespace {

int launch_rc() { return hipGetLastError() == hipSuccess ? ERNIE_OK : ERNIE_EHIP; }

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" {

int ernie_vocab_count(const int32_t* ids_dev, int64_t n, int32_t vocab_full, uint64_t* counts_dev, void* stream) {
  if (vocab_full < 1 || vocab_full > ERNIE_VOCAB_MAX || n < 0 || n > ((int64_t)1 << 39)) return ERNIE_EINVAL;
  if (!counts_dev || !aligned(counts_dev, 8)) return ERNIE_EINVAL;
  if (n == 0) return ERNIE_OK;
  if (!ids_dev || !aligned(ids_dev, 4)) return ERNIE_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // one workgroup per CU at most (each flushes its whole histogram at the end), each with at least 32 KiB of
  // stream; n <= 2^39 keeps a workgroup below 2^32 tokens
  const int64_t per_wg = (int64_t)kCountThreads * 4 * 2;
  const int grid = (int)std::min<int64_t>(256, std::max<int64_t>(1, (n + per_wg - 1) / per_wg));
  if (vocab_full <= kCountMaxLdsVocab) {
    const size_t lds = (size_t)vocab_full * sizeof(unsigned int);
    static bool configured = false;     // raises the dynamic LDS limit once per process (same value for every device)
    if (!configured) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(vocab_count_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              kCountMaxLdsVocab * (int)sizeof(unsigned int)) != hipSuccess)
        return ERNIE_EHIP;
      configured = true;
    }
    hipLaunchKernelGGL(vocab_count_kernel<true>, dim3(grid), dim3(kCountThreads), lds, s, ids_dev, (long long)n,
                       vocab_full, reinterpret_cast<u64_t*>(counts_dev));
  } else {
    hipLaunchKernelGGL(vocab_count_kernel<false>, dim3(grid), dim3(kCountThreads), 0, s, ids_dev, (long long)n,
                       vocab_full, reinterpret_cast<u64_t*>(counts_dev));
  }
  return launch_rc();
}

int ernie_vocab_select(const uint64_t* counts_dev, int32_t vocab_full, int32_t k, const int32_t* reserved_host,
                       int32_t n_reserved, int32_t unk_full_id, int32_t* kept_ids_dev, int32_t* full_to_trimmed_dev,
                       void* stream) {
  if (vocab_full < 1 || vocab_full > ERNIE_VOCAB_MAX || k < 1 || k > vocab_full) return ERNIE_EINVAL;
  if (!counts_dev || !kept_ids_dev || !full_to_trimmed_dev || !reserved_host) return ERNIE_EINVAL;
  if (n_reserved < 1 || n_reserved > ERNIE_VOCAB_MAX_RESERVED || n_reserved > k) return ERNIE_EINVAL;
  ReservedIds res{};
  res.n = n_reserved;
  bool has_unk = false;
  for (int i = 0; i < n_reserved; ++i) {
    const int r = reserved_host[i];
    if (r < 0 || r >= vocab_full) return ERNIE_EINVAL;
    for (int j = 0; j < i; ++j)
      if (res.id[j] == r) return ERNIE_EINVAL;
    res.id[i] = r;
    has_unk |= (r == unk_full_id);
  }
  if (!has_unk) return ERNIE_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // ranks accumulate in the map buffer: zero it, add the partial ranks of every id slice, then compact
  const int blocks = (vocab_full + kRankThreads - 1) / kRankThreads;
  const int tiles = (vocab_full + kRankTile - 1) / kRankTile;
  const int slices = std::max(1, std::min(tiles, 2048 / blocks));
  hipLaunchKernelGGL(fill_int_kernel, dim3((vocab_full + 255) / 256), dim3(256), 0, s, full_to_trimmed_dev, vocab_full, 0);
  hipLaunchKernelGGL(vocab_rank_kernel, dim3(blocks, slices), dim3(kRankThreads), 0, s,
                     reinterpret_cast<const u64_t*>(counts_dev), vocab_full, res, full_to_trimmed_dev);
  hipLaunchKernelGGL(vocab_compact_kernel, dim3(1), dim3(kCompactThreads), 0, s, full_to_trimmed_dev, vocab_full, k,
                     unk_full_id, kept_ids_dev);
  return launch_rc();
}

int ernie_vocab_gather_rows(const void* table_full_dev, int32_t vocab_full, int32_t d, const int32_t* kept_ids_dev,
                            int32_t k, void* table_kept_dev, void* stream) {
  if (!table_full_dev || !kept_ids_dev || !table_kept_dev) return ERNIE_EINVAL;
  if (vocab_full < 1 || k < 1 || d < 8 || d % 8 != 0) return ERNIE_EINVAL;
  if (!aligned(table_full_dev, 16) || !aligned(table_kept_dev, 16)) return ERNIE_EINVAL;
  const int d8 = d / 8;
  const long long total = (long long)k * d8;
  const int grid = (int)std::min<long long>(4096, (total + 255) / 256);
  hipLaunchKernelGGL(vocab_gather_rows_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const int4*>(table_full_dev), vocab_full, d8, kept_ids_dev, k,
                     static_cast<int4*>(table_kept_dev));
  return launch_rc();
}

int ernie_remap_ids(const int32_t* in_dev, int64_t n, const int32_t* map_dev, int32_t map_len, int32_t fallback,
                    int32_t* out_dev, void* stream) {
  if (n < 0 || map_len < 1 || !map_dev) return ERNIE_EINVAL;
  if (n == 0) return ERNIE_OK;
  if (!in_dev || !out_dev || !aligned(in_dev, 4) || !aligned(out_dev, 4)) return ERNIE_EINVAL;
  const int vec_ok = aligned(in_dev, 16) && aligned(out_dev, 16);
  const int grid = (int)std::min<int64_t>(4096, (n / (vec_ok ? 4 : 1) + 255) / 256 + 1);
  hipLaunchKernelGGL(remap_ids_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), in_dev, (long long)n,
                     map_dev, map_len, fallback, out_dev, vec_ok);
  return launch_rc();
}

}  // extern "C"
