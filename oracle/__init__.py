"""CPU oracle for the Contextual Token Sparsity hot path (LeMo, arXiv 2501.09767).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this; it exists so that the
HIP path can be compared, element by element, with a plain fp64 statement of the paper's
definitions (Sec. 4.2 Eq. 1-2 for scoring, Sec. 4.4 for selective load and in-place add).

The arithmetic lives in ``lemo_oracle.c`` (plain C, OpenMP over independent heads / rows); this
module only compiles it with gcc and marshals numpy arrays into it.
"""
from .lemo_oracle import (  # noqa: F401
    BF16, F32, CAUSAL, EXCLUDE_SELF, SCATTER_ACCUMULATE, SCATTER_ZERO_PAD,
    build, num_threads, keep_k, kept_count, score, score_bruteforce, score_blocks, score_block_rows, select_threshold, threshold_init,
    PROBABILITIES, POSITIVE_LOGITS, select_topk, gather_gemm, gather_gemm_add, gather_gemm_dw, kept_attention, scatter_add,
    double_to_bf16_bits, bf16_bits_to_float32, float32_to_bf16_bits,
)
