"""MI355X (gfx950) ERNIE / UNIMO-text generation hot path: C-ABI HIP library + thin binding."""
from .binding import (ErnieConfig, ErnieWeights, ErnieVariants, ernie_init_weights_ex, ErnieEngine, ErnieError, engine_from_workload, load_library,
                      ernie_init_weights, ernie_prefill, ernie_decode_step, ernie_decode_step_static, ernie_last_error, ernie_debug_handover, ernie_free, error_string, EXPORTS,
                      ernie_get_config, ernie_job_workspace_bytes, ernie_run_job, ErnieJob, ErnieJobStats,
                      ernie_set_eos, ernie_batch_state, ernie_compact, ernie_plan_batches,
                      ernie_vocab_count, ernie_vocab_select, ernie_vocab_gather_rows, ernie_remap_ids, VocabTrimmer,
                      ERNIE_OK, ERNIE_EINVAL, ERNIE_ECAPACITY, ERNIE_EARENA, ERNIE_ESEQUENCE, ERNIE_EHIP)
