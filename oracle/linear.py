"""CPU oracle of the linear modules (the other main contributor to a layer's computation time next to
self-attention; Sec. 4.2 "Computation Profiler": the input of dimension (b, S/s_sp, H) applied to a Linear
module), forward and backward.

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the cpu_baseline leg of bench.py.  Nothing on the
product path may import it, and it imports nothing from the product package.

A Linear module without bias (the models of Table 2 are LLaMA-style) with weight w [N, K] ("out, in") maps
x [M, K] (M = b * S/s_sp tokens) to
    y  = x w^T                 [M, N]
and its backward pass, given dy [M, N], returns
    dx = dy w                  [M, K]
    dw = dy^T x                [N, K]
Inputs are the bf16 values the GPU gets, widened exactly to float64; the products are numpy's float64
matmul (a library primitive serving as one step); nothing is rounded.
"""
import numpy as np


def _f64(a):
    a = np.asarray(a)
    assert a.dtype == np.float64, "widen the bf16 inputs to float64 first"
    return a


def linear_fwd(x, w):
    return _f64(x) @ _f64(w).T


def linear_bwd_input(dy, w):
    return _f64(dy) @ _f64(w)


def linear_bwd_weight(dy, x):
    return _f64(dy).T @ _f64(x)
