"""MI355X (gfx950) graph-embedding training step: thin binding over libmarius_hip.so.

The library is loaded on first use; importing the package needs no GPU.
"""
from .binding import (MarConfig, MarDebugOut, MODEL_DISTMULT, MODEL_COMPLEX, MODEL_TRANSE, MODEL_DOT, PRECISION_FP32, PRECISION_SPLIT_BF16, NUM_PHASES,   # noqa: F401
                      MarError, load_library, library_path, mar_workspace_bytes, mar_init_tables,
                      mar_sample_negatives, mar_train_batch, mar_eval_scores, mar_eval_filter, mar_rank_metrics, mar_rank_metrics_static,
                      mar_beta_buffer_sequence,
                      mar_beta_edge_bucket_order, mar_buffer_simulate, mar_swap_lower_bound, mar_beta_swap_count,
                      mar_pipe_workspace_bytes, mar_pipe_create, mar_pipe_submit, mar_pipe_drain, mar_pipe_destroy,
                      mar_profile_enable,
                      mar_profile_read, mar_destroy, mar_last_error, Trainer)
