/*
 * ernie.h -- C ABI of the MI355X (gfx950) ERNIE / UNIMO-text generation hot path.
 *
 * What the library computes (paper: Method, "Model-level optimization"):
 * the FP16 forward of a stack of transformer layers with multi-head
 * self-attention and feed-forward blocks, run as ONE prefill pass over the
 * prompts plus one incremental decode step per generated token that reuses
 * the cached keys and values of all earlier positions (item 3, "Key-Value
 * cache"), followed by the output projection onto the word-embedding matrix
 * trimmed to its frequently used rows ("Embedding layer pruning") and a greedy
 * argmax.  The prompt is attended bidirectionally, generated tokens causally.
 *
 * Conventions common to every entry point
 *  - All pointers named *_dev are DEVICE pointers, *_host are HOST pointers.
 *  - Parameters and activations are IEEE fp16, row-major; accumulation, softmax
 *    and LayerNorm statistics are fp32; logits and hidden outputs are fp32;
 *    token ids are int32 in TRIMMED index space [0, vocab_kept).  The caller
 *    converts to full-vocabulary ids with kept_ids[] (host post-processing).
 *    Ids outside [0, vocab_kept) are not diagnosed on the device: they are clamped into the table (a valid row is
 *    read, never memory past it).
 *  - The caller owns every buffer: parameters, the arena, inputs, outputs, and
 *    the stream.  The library calls no hipMalloc / hipFree in prefill or decode
 *    and enqueues all work on `stream` (a hipStream_t passed as void*; NULL =
 *    the default stream) without synchronising the host, so outputs are valid
 *    once the caller has synchronised the stream.
 *  - A handle is not thread-safe and carries one in-flight batch.
 *  - Test and measurement hooks (ernie_debug_*, ernie_profile*) are declared in ernie_debug.h.
 *  - Return value: 0 on success, a negative ERNIE_E* code otherwise.  Codes
 *    -1..-4 are decided on the host before anything is enqueued and leave the
 *    handle's state unchanged.
 */
#ifndef ERNIE_H_
#define ERNIE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility: only what carries ERNIE_API is exported. */
#define ERNIE_API __attribute__((visibility("default")))

#define ERNIE_OK          0
#define ERNIE_EINVAL     (-1)  /* NULL / misaligned pointer, unsupported shape, length out of range */
#define ERNIE_ECAPACITY  (-2)  /* batch, sequence or position beyond the configured capacity */
#define ERNIE_EARENA     (-3)  /* arena too small (*arena_needed is set) */
#define ERNIE_ESEQUENCE  (-4)  /* decode step before a prefill */
#define ERNIE_EHIP       (-5)  /* HIP runtime error while enqueueing */

typedef struct ErnieHandle ErnieHandle;   /* opaque, library-owned host object */

/* Static shape and capacity.  head_dim = d_model / n_heads must be 64 and
 * d_ffn a multiple of 64.  The key/value cache (Method item 3) holds
 * max_batch sequences of max_seq positions each (prompt + generated). */
typedef struct {
  int32_t n_layers, d_model, n_heads, d_ffn;
  int32_t vocab_full, vocab_kept, max_pos;   /* V, V' (rows of the trimmed table), rows of the position table */
  int32_t max_batch, max_seq;
  float   ln_eps;
} ErnieConfig;

/* Caller-owned DEVICE tensors, fp16 row-major.  Matrices are stored
 * [out, in].  The six/eight per-layer arrays of pointers live on the HOST and
 * have n_layers entries each.
 *   tok_emb_kept [V', d]  rows kept_ids[i] of the full word-embedding matrix;
 *                         used for the input gather AND the output projection
 *   kept_ids     [V']     ascending full-vocabulary ids (int32); stored, not used on the hot path
 *   pos_emb      [P, d]
 *   wqkv[l]      [3d, d]  rows 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V; head h = rows 64h..64h+63 of each block
 */
typedef struct {
  const void*    tok_emb_kept;
  const int32_t* kept_ids;
  const void*    pos_emb;
  const void*    emb_ln_g;  const void* emb_ln_b;      /* [d] */
  const void* const* wqkv;  const void* const* bqkv;   /* [3d, d], [3d] */
  const void* const* wo;    const void* const* bo;     /* [d, d],  [d]  */
  const void* const* ln1_g; const void* const* ln1_b;  /* [d] */
  const void* const* w1;    const void* const* b1;     /* [f, d],  [f]  */
  const void* const* w2;    const void* const* b2;     /* [d, f],  [d]  */
  const void* const* ln2_g; const void* const* ln2_b;  /* [d] */
} ErnieWeights;

/*
 * ernie_init_weights -- size the arena, or ingest the parameters.
 *
 * With arena_dev == NULL: validates cfg, writes the number of bytes the
 * library needs (repacked parameters + key/value cache + activations) to
 * *arena_needed and returns ERNIE_OK; `weights` and `out` may be NULL.
 *
 * With an arena: additionally repacks every parameter into it (the trimmed
 * word-embedding matrix of "Embedding layer pruning" is kept both row-major
 * for the input gather and tiled for the output projection), so the caller's
 * originals may be freed once `stream` has been synchronised, and returns a
 * handle in *out.  arena_dev must be 256-byte aligned; its contents belong to
 * the library until ernie_free.
 *
 * Errors: ERNIE_EINVAL (NULL cfg/out/weight pointer, head_dim != 64,
 * non-positive sizes, misaligned arena), ERNIE_EARENA, ERNIE_EHIP.
 */
ERNIE_API int ernie_init_weights(const ErnieConfig* cfg, const ErnieWeights* weights,
                       void* arena_dev, size_t arena_bytes, size_t* arena_needed,
                       void* stream, ErnieHandle** out);

/*
 * Optional model variants, absent from the paper's description (Method: stacked transformer
 * layers, trimmed word-embedding matrix) but present in public ERNIE / UNIMO checkpoints.
 * Every field may be NULL (variant off); all are caller-owned DEVICE tensors, fp16.
 *   type_emb   [2, d]  segment embedding added to token + position before the embedding
 *                      LayerNorm: row 0 at prompt positions, row 1 at generated positions
 *   head_w     [d, d]  output-head transform t = LayerNorm(gelu(head_w h + head_b)) applied to
 *   head_b, head_ln_g, head_ln_b [d]   the final hidden state before the tied projection;
 *                      all four are required together
 *   out_bias   [V']    added to the logits, already gathered to the KEPT rows (bias_full[kept_ids])
 * hidden_out of prefill / decode stays the final hidden state BEFORE the head transform.
 */
typedef struct {
  const void* type_emb;
  const void* head_w; const void* head_b; const void* head_ln_g; const void* head_ln_b;
  const void* out_bias;
} ErnieVariants;

/*
 * ernie_init_weights_ex -- ernie_init_weights for a model with optional variants.
 * `variants` may be NULL (then identical to ernie_init_weights).  For the size query
 * (arena_dev == NULL) only the NULL-ness of the fields is inspected; the arena grows by
 * the repacked variant parameters.  Additional error: ERNIE_EINVAL if only some of the
 * four head parameters are given.
 */
ERNIE_API int ernie_init_weights_ex(const ErnieConfig* cfg, const ErnieWeights* weights, const ErnieVariants* variants,
                          void* arena_dev, size_t arena_bytes, size_t* arena_needed,
                          void* stream, ErnieHandle** out);

/*
 * ernie_prefill -- one pass over a batch of prompts (FP16 forward, Method
 * item 1; fills the key/value cache of Method item 3) and emission of the
 * first generated token of every sequence from its last prompt position.
 *
 *   B, Lmax            batch size and row pitch of ids_dev
 *   ids_dev            [B, Lmax] trimmed-index prompt ids, right-padded (pad values are ignored)
 *   prompt_lens_host   [B], 1 <= L_b <= Lmax; read before the call returns
 *   logits_out_dev     [B, V'] fp32 logits over the trimmed table, or NULL
 *   hidden_out_dev     [B, d]  fp32 final hidden state at the emitting position, or NULL
 *   tok_out_dev        [B]     int32 argmax (lowest index on exact ties), never NULL
 *
 * Resets the cache: sequence b then holds L_b positions.  Padded positions
 * are never visible as keys.
 * The lengths reach the device through library-owned pinned memory.  Eager calls
 * may follow each other without synchronisation (the call blocks only if the
 * device is eight such copies behind).  A call captured into a graph bakes the
 * lengths of capture time into the graph; its pinned copy stays valid for every
 * replay until ernie_free, and a handle has room for eight captured calls of
 * ernie_prefill / ernie_compact (then ERNIE_ECAPACITY).
 * Errors: ERNIE_EINVAL, ERNIE_ECAPACITY (B > max_batch, Lmax > max_seq,
 * Lmax > max_pos, capture slots used up), ERNIE_EHIP.
 */
ERNIE_API int ernie_prefill(ErnieHandle* h, int32_t B, int32_t Lmax,
                  const int32_t* ids_dev, const int32_t* prompt_lens_host,
                  float* logits_out_dev, float* hidden_out_dev, int32_t* tok_out_dev,
                  void* stream);

/*
 * ernie_decode_step -- one incremental step for every sequence of the batch
 * last given to ernie_prefill: embeds one token per sequence at its next
 * position, appends its key and value to the cache, attends over everything
 * cached (Method item 3: earlier keys/values are read, not recomputed), and
 * emits the next token.
 *
 *   tok_in_dev   [B] trimmed ids to feed (teacher forcing), or NULL to feed
 *                the tokens the previous call emitted (free-running; they are
 *                kept on the device, no host round trip)
 *   outputs      as in ernie_prefill
 *
 * The per-sequence lengths live on the device and advance by one per call, so
 * a stream capture of this call can be replayed.  The host-side capacity check
 * counts calls made through this function only; a replayed capture that runs
 * past max_seq or max_pos makes the kernels skip the step for that sequence
 * instead of writing out of bounds.
 * Errors: ERNIE_ESEQUENCE (no prefill yet), ERNIE_ECAPACITY (some sequence
 * would exceed max_seq or max_pos), ERNIE_EINVAL, ERNIE_EHIP (enqueueing failed, or
 * an EARLIER step's kernel gave up a bounded wait: see ernie_last_error).
 */
ERNIE_API int ernie_decode_step(ErnieHandle* h, const int32_t* tok_in_dev,
                      float* logits_out_dev, float* hidden_out_dev, int32_t* tok_out_dev,
                      void* stream);

/*
 * ernie_last_error -- device-side failures that cannot be reported by the call that enqueued the work.
 * At batch <= 64 the layers of a decode step run as one persistent kernel whose workgroups hand activations to
 * each other through device memory; every wait of that kernel is bounded, and a wait that gives up (which needs
 * a workgroup that is never scheduled, e.g. a GPU shared with another long-running kernel) writes an error
 * word and ends the kernel; the step's outputs are then undefined.  This call returns ERNIE_EHIP once if that
 * has happened since the last report, ERNIE_OK otherwise; the caller synchronises the stream first to be sure
 * the step in question has run.  The next ernie_decode_step reports (and clears) the same condition itself.
 * Error: ERNIE_EINVAL (NULL handle).
 */
ERNIE_API int ernie_last_error(ErnieHandle* h);

/*
 * ernie_decode_step_static -- ernie_decode_step for callers that must not touch an allocator and want the
 * step's temporaries out of their arena: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and errors as ernie_decode_step.  The temporaries of the step
 * (raw fp32 GEMM outputs, fp16 activations, argmax candidates) live in a 5.25 MiB array of static device
 * memory inside the library instead of in the arena; weights, the key/value cache and the per-sequence state
 * stay in the arena.  Each GPU the library runs on holds its own copy of that array until the process ends.
 * Limits (ERNIE_ECAPACITY beyond them, decided on the host before anything is enqueued): batch in flight <= 64,
 * d_model <= 1024, d_ffn <= 4096, vocab_kept <= 32768, and a shape the small-batch decode path accepts.
 * Every call on one GPU uses the same array, whichever handle it is made through: calls that overlap on one GPU
 * (two streams, two handles) race; calls on one stream are ordered and safe.  Nothing in the array has to be
 * zero at entry (every element is written before it is read within a step), so a call after a larger or a
 * smaller batch needs no clearing.  Calls no hipMalloc / hipFree and no allocating library routine.
 */
ERNIE_API int ernie_decode_step_static(ErnieHandle* h, const int32_t* tok_in_dev,
                             float* logits_out_dev, float* hidden_out_dev, int32_t* tok_out_dev,
                             void* stream);

/*
 * End of sequence, batch compaction and batching order.  The paper orders its inputs
 * before inference and lets the batch size follow the input sizes (Introduction; Related
 * work, "Dynamic Batch Size") without giving a procedure; these entry points are the
 * mechanism a caller needs for both.
 *
 * ernie_set_eos -- eos_id is a trimmed id in [0, vocab_kept), or -1 (default) for none.
 * With an id set, a sequence that is FED that id by a decode step (the token it emitted in
 * free-running mode, tok_in_dev[b] under teacher forcing) is finished from that step on:
 * its cache is neither read nor extended, its length stops advancing and it emits eos_id
 * at every later step; its logits / hidden output rows are unspecified.  Other sequences
 * are unaffected.  A prefill clears all finished flags.  Error: ERNIE_EINVAL (id out of range).
 *
 * ernie_batch_state -- copies the per-sequence cached lengths and finished flags (0 / 1) of
 * the current batch into caller buffers of B int32 each (either may be NULL), on `stream`.
 *
 * ernie_compact -- drops sequences from the batch in flight: row i of the new batch is old
 * row keep_rows_host[i] (strictly ascending, n_keep >= 1 of them, read before the call
 * returns).  Cache contents do not move (rows are reached through a device-side row map);
 * later decode steps run with B = n_keep and their outputs have n_keep rows.  A captured
 * graph of decode steps is tied to the batch size it was captured with.
 * Errors: ERNIE_ESEQUENCE (no prefill yet), ERNIE_EINVAL (bad list), ERNIE_ECAPACITY (captured
 * call, capture slots used up: see ernie_prefill), ERNIE_EHIP.
 *
 * ernie_plan_batches -- host-only: orders n requests by prompt length (ascending, equal
 * lengths in arrival order) and cuts the order greedily into batches of at most max_batch
 * rows and at most max_tokens padded tokens (rows x longest prompt of the batch).
 *   order_out_host [n], starts_out_host [n + 1] (the first *n_batches_out + 1 entries are
 *   the cut points into order_out_host).  Error: ERNIE_EINVAL (NULL pointer, n < 0,
 *   limits < 1, a length < 1 or a prompt that alone exceeds max_tokens).
 */
ERNIE_API int ernie_set_eos(ErnieHandle* h, int32_t eos_id);
ERNIE_API int ernie_batch_state(ErnieHandle* h, int32_t* lens_out_dev, int32_t* finished_out_dev, void* stream);
ERNIE_API int ernie_compact(ErnieHandle* h, int32_t n_keep, const int32_t* keep_rows_host, void* stream);
ERNIE_API int ernie_plan_batches(const int32_t* lens_host, int32_t n, int32_t max_batch, int64_t max_tokens,
                       int32_t* order_out_host, int32_t* starts_out_host, int32_t* n_batches_out);

/* ernie_free -- releases the host-side handle (the arena stays the caller's). NULL is a no-op. */
ERNIE_API void ernie_free(ErnieHandle* h);

/* ernie_error_string -- static description of an ERNIE_E* code. */
ERNIE_API const char* ernie_error_string(int code);

#ifdef __cplusplus
}
#endif
#endif  /* ERNIE_H_ */
