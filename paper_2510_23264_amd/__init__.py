"""MI355X-native PAHQ / ACDC edge-ablation path: thin Python binding over libpahq.so."""
from .binding import (lib, PahqError, Config, Model, n_senders, n_receivers, n_upstream, edge_count, edge_id,
                      node_of_receiver, workspace_bytes, measure_ceilings, quantize_rows_noalloc, tau_grid, TraceRec,
                      ALL_FP32, ALL_FP8, PAHQ, MMA_FP8, MMA_F16_EXACT, METRIC_KL, METRIC_LOGIT_DIFF, W_Q, W_K, W_V, W_O, W_IN, W_GATE, W_OUT, W_U)
