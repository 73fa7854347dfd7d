"""CPU oracle for the sliced transformer-block forward, the Step Rehash test and walks, and the
Spatial ResBlock operator group with its Up/DownSample.

TEST INFRASTRUCTURE ONLY.  Plain NumPy in float64, full tensors, one operator
after the other, no blocking or fusion.  Nothing here is imported by the HIP
product path; only the tests, the smoke check and the benchmark's CPU-baseline
leg call it.  It shares no code with the HIP kernels.

Pinned by tests/test_oracle_*.py against closed forms, invariants and an
independent brute-force evaluation.  Not pinned ("parity unpinned"): the
paper's similarity regimes and key-step counts on trained models (Appendix B)
and its end-to-end memory / latency table (Table 1) -- they need trained
weights and video data and are context only.
"""
from .block_ref import (  # noqa: F401
    group_norm_ref, layer_norm_ref, sinusoidal_pe_ref, gelu_erf_ref, softmax_rows_ref,
    attention_ref, tokens_from_feature_ref, feature_from_tokens_ref, transformer_ref,
    block_forward_ref, sliced_block_forward_ref, slice_windows_ref,
)
from .rehash_ref import (  # noqa: F401
    cosine_terms_ref, cosine_ref, rehash_decision_ref, key_step_search_ref, rehash_replay_ref,
    rehash_causal_ref,
)
from .resblock_ref import (  # noqa: F401
    silu_ref, conv3x3_ref, resblock_forward_ref, sliced_resblock_forward_ref,
    downsample_ref, upsample_ref, sliced_resample_ref,
)
