"""CPU oracle for the multi-head speculative decoding step.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 numpy
implementation of what the HIP library computes, written from the paper
(Sec. 4.1-4.2, Eq. 3-4, Alg. 1).  Only the test-suite, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and it
shares no code with the HIP kernels or their Python binding.
"""
from .philox import philox4x32_10, uniform24
from .xsm_oracle import (Oracle, SeqState, VerifyParams, rmsnorm, rope_rotate, gelu_erf, silu,
                         softmax, accept, sample, rank_of, pts_sample, PTS_HEAD)

__all__ = ["philox4x32_10", "uniform24", "Oracle", "SeqState", "VerifyParams", "rmsnorm",
           "rope_rotate", "gelu_erf", "silu", "softmax", "accept", "sample", "rank_of", "pts_sample",
           "PTS_HEAD"]
