/*
 * ernie_job.h -- C ABI of the host pipeline around the generation hot path
 * (paper: Method, "Multi-process parallel processing": serving is split into a
 * main, a preprocessing, a model-inference and a post-processing worker that run
 * side by side instead of one after another).
 *
 * ernie_run_job takes a list of requests (prompts in FULL-vocabulary ids, on the
 * host), and
 *   main            orders them by length and cuts them into batches (ernie_plan_batches),
 *   preprocessing   re-indexes each batch to trimmed ids and right-pads it into pinned memory,
 *   inference       uploads the batch and enqueues one prefill + n_gen - 1 free-running
 *                   decode steps (ernie_prefill / ernie_decode_step) and the download of the tokens,
 *   post-processing waits for the batch, maps the tokens back to full ids and stores them in
 *                   request order.
 * With overlap = 1 the three workers are threads over two batch slots, so the GPU is
 * handed batch i + 1 while batch i is still running and batch i - 1 is being written out;
 * with overlap = 0 the same stage functions run one after another in the calling thread.
 * Both give bit-identical results.
 *
 * Pointers named *_host are HOST pointers, *_dev DEVICE pointers; the caller owns all of
 * them.  The call allocates pinned host staging (hipHostMalloc) and events, frees them
 * before it returns, and returns when every request is done.  Return codes as in ernie.h.
 */
#ifndef ERNIE_JOB_H_
#define ERNIE_JOB_H_

#include <stddef.h>
#include <stdint.h>

#include "ernie.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t n_requests;
  const int32_t* prompt_offsets_host;    /* [n_requests + 1] ascending offsets into prompt_ids_host; every prompt has >= 1 id */
  const int32_t* prompt_ids_host;        /* full-vocabulary ids in [0, vocab_full) */
  const int32_t* full_to_trimmed_host;   /* [vocab_full] trimmed index of every full id (dropped ids: the unknown-word row) */
  const int32_t* kept_ids_host;          /* [vocab_kept] full id of every trimmed index */
  int32_t n_gen;                         /* tokens to generate per request, >= 1 */
  int32_t max_batch;                     /* rows per batch, 1 .. the handle's max_batch */
  int64_t max_tokens;                    /* padded prompt tokens per batch (rows x longest prompt) */
  int32_t overlap;                       /* 0 = stages one after another, 1 = stages side by side */
  void*   workspace_dev;                 /* >= ernie_job_workspace_bytes(h, n_gen), 256-byte aligned */
  size_t  workspace_bytes;
  int32_t* tokens_out_host;              /* [n_requests, n_gen] generated FULL ids, request order */
} ErnieJob;

typedef struct {
  double pre_s, enqueue_s, post_s;       /* busy time of the three workers (post_s excludes waiting for the GPU) */
  double wall_s;                         /* whole call */
  int32_t n_batches;
} ErnieJobStats;

/* ernie_get_config -- copies the configuration the handle was created with. */
ERNIE_API int ernie_get_config(const ErnieHandle* h, ErnieConfig* out);

/* Device workspace of a job: two batch slots of padded prompt ids and generated tokens. 0 if h is NULL or n_gen < 1. */
ERNIE_API size_t ernie_job_workspace_bytes(const ErnieHandle* h, int32_t n_gen);

/*
 * ernie_run_job -- see the top of this file.  `stats_out` may be NULL.
 * Errors, all decided before any work is enqueued: ERNIE_EINVAL (NULL pointer, offsets not
 * ascending, an id outside [0, vocab_full) or a map entry outside [0, vocab_kept), limits
 * < 1, workspace too small or misaligned), ERNIE_ECAPACITY (max_batch beyond the handle's, a
 * prompt whose length + n_gen - 1 exceeds max_seq or max_pos).  ERNIE_EHIP if a HIP call fails
 * while running (remaining batches are abandoned; tokens_out_host is then incomplete).
 */
ERNIE_API int ernie_run_job(ErnieHandle* h, const ErnieJob* job, ErnieJobStats* stats_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif  /* ERNIE_JOB_H_ */
