"""MI355X-native hot path of Activation Subspace Iteration (arxiv 2505.05086).

Thin Python names over the C ABI of libasi_hip.so (see include/asi.h):
asi_compress, asi_core_project, asi_weight_grad_conv2d, asi_weight_grad_linear and their
*_batch forms, which serve several layers with every kernel launch; asi_compress_cold for the first
iteration; AsiConv2d / AsiLinear wire the calls into autograd (the layers keep (S, U), not the activation);
rank_selection holds the front end of Sec. 3.3 (mode spectra, explained-variance ranks, perplexity rows, the
budgeted choice).
"""
from .autograd import AsiConv2d, AsiLinear, AsiState  # noqa: F401
from .binding import (  # noqa: F401
    ASI_BF16,
    ASI_F32,
    AsiError,
    Conv2dDesc,
    EXPORTS,
    TensorDesc,
    alloc_workspace,
    asi_activation_memory,
    asi_compress,
    asi_cold_start_matrix,
    asi_compress_batch,
    asi_compress_cold,
    asi_compress_static,
    asi_core_project,
    asi_core_project_batch,
    asi_explained_variance_ranks,
    asi_frobenius_diff,
    asi_mode_spectrum,
    asi_mode_spectrum_workspace_bytes,
    asi_profile_enable,
    asi_profile_report,
    asi_rank_select,
    asi_status_string,
    asi_version,
    asi_weight_grad_conv2d,
    asi_weight_grad_conv2d_batch,
    asi_weight_grad_linear,
    asi_weight_grad_linear_batch,
    asi_workspace_bytes,
    lib,
    make_conv,
    make_desc,
)
from . import rank_selection  # noqa: F401,E402
