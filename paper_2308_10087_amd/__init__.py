"""gnnstage: one pipeline stage of chunk-based pipelined GNN training on one MI355X.

The work is done by hand-written HIP kernels in ``libgnnstage.so`` (C ABI declared in
``include/gnnstage.h``); this package only marshals arguments.  There is no CPU fallback:
importing :mod:`binding` raises if the library has not been built.
"""
from .binding import (  # noqa: F401
    GNNSTAGE_BF16, GNNSTAGE_F32, GNNSTAGE_GCN, GNNSTAGE_GCNII, GNNSTAGE_RESGCN, GNNSTAGE_SAGE, GnnStage, GnnStageError, KIND_NAMES,
    gnnstage_dense_plan, gnnstage_plan_pack, gnnstage_plan_tasks, gnnstage_plan_transpose, gnnstage_version, lib,
    GNNTRAIN_ADAM, GNNTRAIN_SGD, GnnTrainer, gnntrain_adam_step, gnntrain_chunk_order, gnntrain_sgd_step,
    gnntrain_softmax_xent, gnntrain_sum, gnntrain_sum_static, gnnstage_partition_chunks, gnnstage_permute_csr,
    gnnstage_debug_gather_rate,
)
