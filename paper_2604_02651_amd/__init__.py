"""MI355X-native hot path of mini-batch GCN training with uniform vertex sampling
(ScaleGNN, arXiv 2604.02651): Python binding of the C library libsgnn.

Every step of the path runs in the hand-written HIP kernels of libsgnn.so; this package only
marshals arguments (torch tensors -> raw device pointers).  There is no CPU fallback: importing
the binding without a built library raises.
"""
from .binding import (  # noqa: F401
    Context, Csr, SgnnError, lib, lib_path,
    SGNN_RELU, SGNN_BF16_MFMA, SGNN_XFORM_FIRST, SGNN_DY_MASKED, SGNN_FUSE_TAIL,
    sgnn_sample_uniform, sgnn_sample_uniform_static, sgnn_induced_csr, sgnn_csr_plan, sgnn_gather_rows, sgnn_gcn_fwd, sgnn_gcn_bwd,
    sgnn_softmax_xent, sgnn_spmm_xent, sgnn_spmm, sgnn_gemm, sgnn_copy_f32, sgnn_tail_fwd, sgnn_tail_bwd, sgnn_gemm_tail_fwd, sgnn_sgd_step, sgnn_adam_step, sgnn_graph_normalized_csr, sgnn_induced_csr_range, sgnn_csr_transpose, sgnn_sigmoid_bce, sgnn_colsum,
)
from .step import GcnStep  # noqa: F401
from .model import ScaleGnnModel  # noqa: F401
