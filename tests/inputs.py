"""INT8 activations for the tests: the shared generator draws FP16 values only, and the
per-token quantisation that turns them into what the GEMM consumes is the oracle's
(Sec. 6 "Serving System"), never the library's."""
from __future__ import annotations

from oracle import lqq_oracle as O
from paper_2509_01229_amd import workloads as WL


def make_activations(M, K, outlier_frac=0.0, seed=0, rng=None):
    """(X_i8 [M,K] int8, s_x [M] float32) of the seeded FP16 draw."""
    return O.quantize_activations(WL.make_activations_f16(M, K, outlier_frac, seed, rng))


def make_problem(shape):
    """(W float32 [N,K] with FP16 values, X_i8 [M,K], s_x [M]) for one workload shape."""
    W, X = WL.make_problem_f16(shape)
    X_i8, s_x = O.quantize_activations(X)
    return W, X_i8, s_x
