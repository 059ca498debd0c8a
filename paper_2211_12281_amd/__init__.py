"""MI355X-native hot path of BESS-style knowledge-graph-embedding training and inference
(arXiv 2211.12281): a C-ABI HIP library (csrc/, include/kge.h) and its thin ctypes binding."""
from .binding import (calibrate_copy, debug_select, calibrate_mfma, Encoder, KgeError, ensemble, Model, TripleSampler, Workspace, load, loss_bwd, partition_triples,  # noqa: F401
                      profile_collect, profile_enable, sample_negatives, sample_negatives_dev, sample_negatives_sharded, score,
                      step_counter_add,
                      sparse_adam, sparse_adam_apply, sparse_adam_apply_tables, sparse_adam_plan, sparse_adam_plan_tables, sparse_adam_static, sparse_adam_static_limit, status_string, topk, workspace_bytes)
