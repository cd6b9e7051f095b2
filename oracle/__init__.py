"""CPU oracle of the DeepSqueeze step (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library and its Python binding never do.
"""
from .ds_oracle import (  # noqa: F401
    KIND_IDENTITY, KIND_QUANT_MAXABS, KIND_SIGN_MEANABS, KIND_TOPK, KIND_QUANT_L2NORM, KIND_RAND_SPARSE, KIND_GSPAR,
    ALGO_DEEPSQUEEZE, ALGO_DCD_PSGD, ALGO_CHOCO_SGD,
    OracleState, build_oracle, philox4x32_10, rounding_word, step, step_window,
    ring_matrix, torus_matrix, dense_to_csr, message_bytes, diagnostics, sum_squares_tree, keep_word, rand_sparse_capacity, threads, gspar_word, sum_abs_tree,
)
