/*
 * ernie_debug.h -- test and measurement hooks of the ERNIE generation library: inspection of internal buffers,
 * per-kernel timing, and the tuning knobs the tests and the benchmark use to force a code path.  None of them is
 * part of the hot path (paper: Method, "Model-level optimization"), and none is needed to use the library; the
 * product interface is ernie.h.  Conventions (pointers, return codes) are those of ernie.h.
 */
#ifndef ERNIE_DEBUG_H_
#define ERNIE_DEBUG_H_

#include "ernie.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * ernie_debug_buffer -- test hook: device address and size in bytes of an
 * internal buffer, for layer-by-layer comparison with a reference.  `name`
 * is one of "x" (layer input/output activations [T, d] fp16), "kv" (the
 * key/value cache [n_layers][2][max_batch][n_heads][max_seq][64] fp16),
 * "lens" ([max_batch] int32 cached lengths), "persist_trace" (the time stamps of the
 * one-launch decode kernel, see the "persist_trace" knob below).  Returns ERNIE_EINVAL for an
 * unknown name.  Not part of the hot path.
 */
ERNIE_API int ernie_debug_buffer(ErnieHandle* h, const char* name, void** ptr_dev, size_t* bytes);

/*
 * ernie_profile / ernie_profile_read -- measurement hooks (not part of the hot path).
 *
 * ernie_profile(h, 1) switches per-kernel timing on and clears the counters: from then on every
 * launch of the categories below is bracketed by HIP events recorded on the stream it is launched
 * on (events are created on the first enable; up to 32768 launches are recorded, later ones are not
 * timed).  Do not capture profiled calls into a graph.  ernie_profile(h, 0) switches it off.
 * ernie_profile_read waits for the recorded events of one category and returns the summed device
 * time between each pair, the number of launches, and the algorithmic bytes and flops of those
 * launches: weight bytes N*K*2 for the decode GEMMs and the output projection, K and V bytes of all
 * visible positions for decode attention, 2*M*N*K flops for GEMMs and 4*sum(L_b^2)*d for prefill
 * attention.
 */
#define ERNIE_PROF_GEMM_DEC      0   /* decode GEMM on fp16 activations (attention output, FFN2) */
#define ERNIE_PROF_GEMM_DEC_LN   1   /* decode GEMM with a LayerNorm prologue (QKV incl. the embedding LayerNorm of layer 0, FFN1) */
#define ERNIE_PROF_ATTN_DEC      2   /* decode attention over the key/value cache */
#define ERNIE_PROF_GEMM_PREFILL  3   /* prefill MFMA GEMMs */
#define ERNIE_PROF_ATTN_PREFILL  4   /* prefill attention */
#define ERNIE_PROF_LOGITS        5   /* output projection + first argmax stage (decode, small-batch path) */
#define ERNIE_PROF_ROW_DEC       6   /* decode row kernels: embedding + LayerNorm, final LayerNorm, second argmax stage */
#define ERNIE_PROF_ROW_PREFILL   7   /* prefill row kernels: token map, embedding + LayerNorm, LayerNorm, last-row gather, argmax */
#define ERNIE_PROF_DEC_PERSIST   8   /* the one-launch decode kernel: every layer of a small-batch step (weights + cache bytes) */
#define ERNIE_PROF_NCAT          9
ERNIE_API int ernie_profile(ErnieHandle* h, int enable);
ERNIE_API int ernie_profile_read(ErnieHandle* h, int category, double* total_ms, int64_t* launches,
                       double* alg_bytes, double* alg_flops);

/*
 * ernie_debug_tune -- test hook: override a decode-path tuning knob of this handle.
 *   "fused_decode" 0/1  use the small-batch path (row-wise work fused into GEMM prologues) when it fits,
 *                       else the large-batch path (split-K partials summed by row kernels)
 *   "sk_out", "sk_f2"   split of the contraction of the attention-output / second FFN GEMM over workgroups
 *   "attn_dec" 0..5     decode attention shape: 0 = chosen from the batch and capacity, 1 = 4 waves x 4 key groups
 *                       in flight, 2 = 8 waves x 3, 3 = 8 waves x 4, 4 = 4 waves x 2, 5 = 2 waves x 2 (a batch of
 *                       waves x groups x 8 keys per memory round trip)
 *   "ln_ns" 0/1/2/4     32-column strips per workgroup of the decode GEMMs with the LayerNorm prologue (0 = chosen
 *                       automatically); "ln_rpw" 0/1/2 rows normalised per wave in that prologue (0 = chosen from the batch size)
 *   "big_logits_gemm" 0/1  large-batch path: output projection on the MFMA GEMM pipeline followed by a row argmax
 *                       (default 1; needs vocab_kept % 8 == 0), or the table-streaming kernel with per-strip argmax
 *   "big_f1_fused" 0/1  large-batch path: first FFN GEMM unsplit with bias + GELU in its epilogue (default 1), or
 *                       split over the contraction with a separate GELU row kernel
 *   "dec_nw16" 0..3     decode GEMMs on fp16 activations with 16 instead of 8 waves per workgroup: 0 = never,
 *                       1 = second FFN GEMM, 2 = also the attention-output GEMM (default), 3 = also the projection
 *   "dec_prefetch" 0..1024  small-batch path: workgroups appended to the attention-output and second FFN GEMMs that
 *                       pull what the next kernel reads first (the weights of the following LayerNorm-prologue GEMM,
 *                       into the L2 of the XCD that will read them, and its bias / scale / shift vectors) out of
 *                       HBM ahead of time (default 64; 0 = off; rounded up to a multiple of 8 per split).  Does
 *                       not change any result.
 *   "kv_prefetch" 0..2048  small-batch path: workgroups appended to the QKV GEMM that stream the cache rows of the
 *                       attention that follows into the L2 of the XCD that will read them (0 = off, 1 = one
 *                       workgroup per two (sequence, head) streams (default), larger = that many workgroups,
 *                       rounded up to a multiple of 8).  Does not change any result.
 *   "big_warm" 0..256   large-batch path: workgroups appended to the decode attention that pull the layer's bias and
 *                       LayerNorm vectors (read first by the row kernels and the FFN1 epilogue that follow) and the
 *                       next layer's QKV bias into every XCD's L2 (default 16; 0 = off).  Does not change any result.
 *   "big_f1_tile" 0..2  large-batch path, first FFN GEMM (unsplit): 0 = 64 x 32 tiles when 64 x 64 ones would number
 *                       128 or fewer, else 64 x 64 (default), 1 = 64 x 32, 2 = 64 x 64.  Does not change any result.
 *   "big_mfast" 0/1     large-batch path: with exactly two row tiles (64 < B <= 128) the tiles of the decode GEMMs are
 *                       ordered rows-fastest, so that both row tiles of a weight column strip run in one XCD and the
 *                       strip is fetched once (default 1).  Does not change any result.
 *   "big_narrow" 0/1    large-batch path: split-K projections whose 64 x 64 tiles times splits number 128 or fewer
 *                       run on 64 x 32 tiles instead (default 1).  Does not change any result.
 *   "big_ln_rows" 1/2/4 large-batch path: rows per workgroup of the LayerNorm row kernels (default 1: a row's
 *                       partial sums are 20 KB at d = 1024, and several rows behind one CU's memory pipeline
 *                       lengthen these short kernels).  Does not change any result.
 *   "pf_tile" 0..3      prefill GEMM tile: 0 = chosen from the problem size (default), 1 = 256 x 256, 2 = 128 x 128,
 *                       3 = 64 x 64.  Does not change any result.
 *   "attn_nt" 0/1       decode attention reads the cache with the non-temporal (streaming) hint, so that the
 *                       once-per-step cache stream does not displace the weights from the caches (default 1)
 *   "persist" 0/1       batch <= 64: all layers of a decode step in one persistent kernel (default 1 where it fits), or
 *                       five kernels per layer
 *   "persist_helpers" 0/1  workgroups of that kernel that own no unit run ahead and pull weights and cache rows into
 *                       the L2 of the XCD that will read them (default 1).  Does not change any result.
 *   "persist_spin" >= 1 polls after which a workgroup of that kernel gives up a wait (default 2^17); the step then
 *                       ends by itself and the next call on the handle returns ERNIE_EHIP
 *   "persist_stall" 0..5  test hook: withhold the output of phase 1..5 (QKV, attention, attention output, FFN1, FFN2)
 *                       of layer 0, so that its consumers' bounded waits give up (0 = off)
 *   "persist_trace" 0/1 every workgroup of that kernel writes 100 MHz time stamps (phase entry, input arrived, output
 *                       published; helpers: wait ended, warm-up landed) into the buffer "persist_trace",
 *                       [workgroup][layer][32] uint64 (see ernie_debug_buffer; slot 31 = bit mask of the phases the workgroup owned
 *                       a unit of); for at most 512 workgroups
 *   "persist_dbg"       measurement hook, bit mask: 1 = helper workgroups idle, 2 = no weight loads (results are
 *                       wrong), 4 = helpers leave the projection table alone; value / 16 = phases the helpers stay
 *                       ahead of the publishing front (0 = default, 3)
 * Splits are 1, 2 or 4.  Results are deterministic for any fixed setting.  Returns ERNIE_EINVAL for an
 * unknown key or a split that is not supported or does not divide the k-tile count.
 */
ERNIE_API int ernie_debug_tune(ErnieHandle* h, const char* key, int value);

/*
 * ernie_debug_handover -- measures what it costs to hand data from every workgroup of a persistent kernel to
 * every other one through device memory, i.e. the price of one phase boundary of the one-launch decode step
 * (paper: Method, "Processing Optimization" counts kernel launches; this is what replaces a launch).
 * n_workgroups workgroups of 512 threads run `stages` dependent stages; per stage each publishes out_units
 * 16-byte units and reads `pieces` (1, 3, 6 or 12) units per thread, spread over all producers.
 *   mode 0  tagged pairs read and written at agent scope (the protocol of the decode kernel)
 *   mode 1  plain stores + release fence + one flag per workgroup; acquire fence + plain loads on the other side
 * ws_dev: caller-owned device workspace, 256-byte aligned, at least 48 * n_workgroups * out_units + 4352 bytes
 * (n_workgroups * out_units must be a multiple of 64); contents are overwritten.  Synchronises `stream`.
 * *us_per_stage = best of four runs; *bad_units = units whose payload was not the expected one (0 for a correct
 * protocol).  Errors: ERNIE_EINVAL (arguments), ERNIE_EHIP (runtime error, or a bounded wait gave up).
 */
ERNIE_API int ernie_debug_handover(int mode, int n_workgroups, int stages, int pieces, int out_units, void* ws_dev,
                                   size_t ws_bytes, void* stream, double* us_per_stage, int64_t* bad_units);

#ifdef __cplusplus
}
#endif
#endif  /* ERNIE_DEBUG_H_ */
