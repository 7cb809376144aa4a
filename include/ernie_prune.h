/*
 * ernie_prune.h -- C ABI of the vocabulary-trimming step that precedes the
 * generation hot path (paper: Method, "Embedding layer pruning": the word-
 * embedding matrix keeps only its frequently used rows).
 *
 * The paper prints no procedure; the library implements the plain one:
 *   ernie_vocab_count   occurrences of every vocabulary id in a token stream
 *   ernie_vocab_select  the k ids to keep (reserved ids first, then higher count,
 *                       then lower id), ascending, plus the full -> trimmed id map
 *   ernie_vocab_gather_rows  the trimmed table = rows kept_ids of the full table
 *   ernie_remap_ids     applies an id map to data (full -> trimmed on the way in,
 *                       trimmed -> full through kept_ids on the way out)
 * All results are exact integers / bit copies.  Every pointer named *_dev is a
 * DEVICE pointer, *_host a HOST pointer; the caller owns all buffers; work is
 * enqueued on `stream` (hipStream_t as void*, NULL = default stream) without a
 * host synchronisation; no entry point allocates.  Return codes are those of
 * ernie.h (0, ERNIE_EINVAL = -1, ERNIE_EHIP = -5); ERNIE_EINVAL is decided on
 * the host before anything is enqueued.
 */
#ifndef ERNIE_PRUNE_H_
#define ERNIE_PRUNE_H_

#include <stddef.h>
#include <stdint.h>

#include "ernie.h"

#ifdef __cplusplus
extern "C" {
#endif

#define ERNIE_VOCAB_MAX        262144   /* largest vocab_full accepted (selection compares all id pairs) */
#define ERNIE_VOCAB_MAX_RESERVED   16

/*
 * ernie_vocab_count -- counts_dev[v] += number of i < n with ids_dev[i] == v.
 *   ids_dev     [n] int32, 4-byte aligned; values outside [0, vocab_full) are ignored
 *   counts_dev  [vocab_full] uint64, 8-byte aligned; ACCUMULATED into, so the caller
 *               zeroes it before the first call and may stream a corpus in pieces
 * n == 0 is a no-op.  Errors: ERNIE_EINVAL (NULL pointer with n > 0, misalignment,
 * vocab_full outside [1, ERNIE_VOCAB_MAX], n < 0 or n > 2^39).
 */
ERNIE_API int ernie_vocab_count(const int32_t* ids_dev, int64_t n, int32_t vocab_full,
                      uint64_t* counts_dev, void* stream);

/*
 * ernie_vocab_select -- chooses the k rows to keep and builds both id maps.
 *   counts_dev           [vocab_full] uint64 (each < 2^63)
 *   reserved_host        [n_reserved] distinct ids kept whatever their count
 *                        (n_reserved <= ERNIE_VOCAB_MAX_RESERVED, <= k); must contain unk_full_id
 *   unk_full_id          the unknown-word id: every dropped id maps to ITS trimmed index
 *   kept_ids_dev         [k] int32 out: kept full ids, ascending (= the trimmed -> full map)
 *   full_to_trimmed_dev  [vocab_full] int32 out: trimmed index of every full id
 * Preference order: reserved ids, then larger count, then smaller id.
 * Errors: ERNIE_EINVAL (NULL pointer, k outside [1, vocab_full], bad or duplicate
 * reserved ids, unk_full_id not reserved, vocab_full outside [1, ERNIE_VOCAB_MAX]).
 */
ERNIE_API int ernie_vocab_select(const uint64_t* counts_dev, int32_t vocab_full, int32_t k,
                       const int32_t* reserved_host, int32_t n_reserved, int32_t unk_full_id,
                       int32_t* kept_ids_dev, int32_t* full_to_trimmed_dev, void* stream);

/*
 * ernie_vocab_gather_rows -- table_kept[i, :] = table_full[kept_ids[i], :], bit for bit.
 *   table_full_dev [vocab_full, d] and table_kept_dev [k, d]: 2-byte elements, row-major,
 *   16-byte aligned, d a multiple of 8; kept ids are not range-checked on the device beyond
 *   being clamped into [0, vocab_full).
 * Errors: ERNIE_EINVAL (NULL pointer, misalignment, d % 8 != 0, non-positive sizes).
 */
ERNIE_API int ernie_vocab_gather_rows(const void* table_full_dev, int32_t vocab_full, int32_t d,
                            const int32_t* kept_ids_dev, int32_t k, void* table_kept_dev, void* stream);

/*
 * ernie_remap_ids -- out[i] = map[in[i]] if 0 <= in[i] < map_len, else fallback.
 *   in_dev, out_dev [n] int32 (may be the same buffer); map_dev [map_len] int32.
 * Errors: ERNIE_EINVAL (NULL pointer with n > 0, misalignment, map_len < 1, n < 0).
 */
ERNIE_API int ernie_remap_ids(const int32_t* in_dev, int64_t n, const int32_t* map_dev, int32_t map_len,
                    int32_t fallback, int32_t* out_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif  /* ERNIE_PRUNE_H_ */
