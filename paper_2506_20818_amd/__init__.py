"""MI355X-native training step for GNN link prediction (one worker of the data-parallel method).

Thin Python binding over the C ABI declared in include/lp.h.  The binding only marshals arguments; every step
runs in the HIP kernels of liblp_mi355x.so.  There is no CPU fallback: importing `binding` without the built
library raises.
"""
from .binding import (  # noqa: F401
    LP_LAYER_GCN,
    LP_LAYER_SAGE_MEAN,
    LP_SYMMETRIZE,
    Acts,
    AdamState,
    BlockActs,
    Blocks,
    Csr,
    Grads,
    LpError,
    Mlp,
    MlpActs,
    MlpGrads,
    Model,
    Sparsified,
    lib_path,
    load_library,
    lp_backward,
    lp_backward_blocks,
    lp_backward_edge_grads,
    lp_mlp_backward,
    lp_mlp_score_loss,
    lp_build_csr,
    lp_adam_step,
    lp_adam_update_tensor,
    lp_sage_forward,
    lp_sage_forward_blocks,
    lp_sample_blocks,
    lp_sgd_step,
    lp_sgd_update_tensor,
    lp_sample_neg,
    lp_score_loss,
    lp_sparsify,
    lp_strerror,
    lp_timing_collect,
    lp_timing_enable,
)
