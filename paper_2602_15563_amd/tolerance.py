"""Acceptance bounds of the parity checks, in one place (tests/ and bench.py use these and nothing else).

Notation: Y the oracle's fp64 result, A = sum_k |w x| the oracle's absolute sum (the contract's tolerance
scale), K the row length.  Everything here is numpy on the oracle's outputs; nothing of the method's
arithmetic lives in this file.

1. TOL: the benchmark contract's criterion, |y_gpu - Y| <= 2e-3 * A.
2. arithmetic_bound: what the arithmetic itself allows for ANY shape.  fp32 accumulation in any order is
   within K * 2^-23 * A of the exact sum, and rounding the result to bf16 (8 significant bits) adds at most
   half an ulp <= 2^-8 * |y|.  For short or same-sign rows |y| is close to A and that rounding alone exceeds
   TOL * A (a single product, K = 1, can be off by 0.39 % of itself in any bf16 output), so the contract's
   criterion is asserted where it is attainable (K >= 512 and all benchmark configurations: long mixed-sign
   sums) and this bound everywhere.
3. swiglu_bound: y = silu(g) * u with g, u two products.  silu' lies in [-0.1, 1.1], so an error dg in g and
   du in u moves y by at most 1.1 |u| dg + |silu(g)| du + 1.1 dg du; the combination itself takes a few fp32
   roundings, and the result one bf16 rounding.
4. rmsnorm_commute_bound: the fused calls' definition rounds x * r * g to bf16; the kernels round x * g and
   apply the scalar r to the fp32 sum.  Both roundings are within half an ulp (2^-8 relative) of the same
   exact value, so an activation differs by at most 2^-7 of itself and the sum by at most 2^-7 * sum |w xn|
   (worst case: both roundings opposed on every term; independent errors add in quadrature, so long rows
   stay far inside TOL * A, which the callers assert as well for K >= 512).
"""
import numpy as np

TOL = 2e-3


def arithmetic_bound(A, Y, K):
    return (K + 8) * 2.0 ** -23 * A + 2.0 ** -8 * (np.abs(Y) + (K + 8) * 2.0 ** -23 * A)


def swiglu_bound(G, U, Ag, Au, silu_G, want, K):
    """G, U: the two fp64 products; Ag, Au: their absolute sums; silu_G = silu(G); want = silu(G) * U."""
    dg, du = (K + 8) * 2.0 ** -23 * Ag, (K + 8) * 2.0 ** -23 * Au
    inner = 1.1 * np.abs(U) * dg + np.abs(silu_G) * du + 1.1 * dg * du + 8 * 2.0 ** -23 * np.abs(want)
    return inner + 2.0 ** -8 * (np.abs(want) + inner)


def swiglu_contract_bound(U, Ag, Au, silu_G, want):
    """The contract's 2e-3 * A on each product, carried through the combination, plus the bf16 rounding."""
    return TOL * (1.1 * np.abs(U) * Ag + np.abs(silu_G) * Au) + 2.0 ** -8 * np.abs(want)


def rmsnorm_commute_bound(A_product):
    """A_product: sum_k |w xn| of the product alone (without a residual)."""
    return 2.0 ** -7 * A_product
