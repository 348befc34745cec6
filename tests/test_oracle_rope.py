"""Pins of the oracle's rotary position embedding (Sec. 3.3) and of its backward.

The paper names the method only (RoFormer); what the oracle computes is pinned against an independent
statement of the same rotation (multiplication by e^{i*angle} of the complex number x0 + i*x1, numpy
complex128), exact special angles, the invariants a rotation has, and the adjoint identity for the backward.
"""
import numpy as np
import pytest

import oracle
from paper_2512_13368_amd.inputs import rope_tables, round_to_bf16


def _x(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def test_rope_is_complex_multiplication():
    L, d = 37, 16
    x = _x((2, 3, L, d), 1)
    cos, sin = rope_tables(L, d)
    got = oracle.rope(x, cos, sin).astype(np.float64)
    z = x[..., 0::2].astype(np.complex128) + 1j * x[..., 1::2].astype(np.complex128)
    w = z * (cos.astype(np.float64) + 1j * sin.astype(np.float64))
    ref = np.empty(x.shape, dtype=np.float64)
    ref[..., 0::2], ref[..., 1::2] = w.real, w.imag
    assert np.max(np.abs(got - ref)) <= 4e-7 * np.max(np.abs(ref))   # two fp32 roundings per element


def test_rope_exact_special_angles():
    L, d = 5, 8
    x = _x((1, 1, L, d), 2)
    one, zero = np.ones((L, d // 2), np.float32), np.zeros((L, d // 2), np.float32)
    np.testing.assert_array_equal(oracle.rope(x, one, zero), x)                       # angle 0: identity
    q = oracle.rope(x, zero, one)                                                    # quarter turn
    np.testing.assert_array_equal(q[..., 0::2], -x[..., 1::2])
    np.testing.assert_array_equal(q[..., 1::2], x[..., 0::2])
    np.testing.assert_array_equal(oracle.rope(x, -one, zero), -x)                     # half turn
    cos, sin = rope_tables(L, d)
    np.testing.assert_array_equal(oracle.rope(x, cos, sin)[..., 0, :], x[..., 0, :])  # position 0 is not rotated


def test_rope_preserves_norms_and_depends_on_relative_position_only():
    L, d = 64, 32
    q, k = _x((1, 1, L, d), 3), _x((1, 1, L, d), 4)
    cos, sin = rope_tables(L, d)
    rq, rk = oracle.rope(q, cos, sin).astype(np.float64), oracle.rope(k, cos, sin).astype(np.float64)
    for a, b in ((q, rq), (k, rk)):   # every channel pair keeps its length
        n0 = a[..., 0::2].astype(np.float64) ** 2 + a[..., 1::2].astype(np.float64) ** 2
        n1 = b[..., 0::2] ** 2 + b[..., 1::2] ** 2
        assert np.max(np.abs(n0 - n1)) <= 1e-6 * np.max(n0)
    # one query vector at positions m and m+t against one key vector at n and n+t: equal inner products
    qq = np.broadcast_to(q[:, :, :1], q.shape).copy()
    kk = np.broadcast_to(k[:, :, :1], k.shape).copy()
    rq, rk = oracle.rope(qq, cos, sin).astype(np.float64)[0, 0], oracle.rope(kk, cos, sin).astype(np.float64)[0, 0]
    S = rq @ rk.T
    for off in (0, 1, 5, 17):
        diag = np.array([S[m + off, m] for m in range(L - off)])
        assert np.max(np.abs(diag - diag[0])) <= 2e-5 * np.abs(S).max()
    assert abs(S[9, 2] - S[2, 9]) > 1e-3 * np.abs(S).max()      # and the sign of the offset matters


def test_rope_bf16_rounding_is_nearest_even():
    L, d = 33, 16
    x = _x((2, 2, L, d), 5)
    cos, sin = rope_tables(L, d)
    full = oracle.rope(x, cos, sin)
    rounded = oracle.rope(x, cos, sin, to_bf16=True)
    np.testing.assert_array_equal(rounded, round_to_bf16(full))   # the input generator's own rounding
    assert np.all((rounded.view(np.uint32) & 0xFFFF) == 0)
    # a tie rounds to the even neighbour: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7
    tie = np.full((1, 1, 1, 2), 1.0 + 2.0 ** -8, np.float32)
    one, zero = np.ones((1, 1), np.float32), np.zeros((1, 1), np.float32)
    np.testing.assert_array_equal(oracle.rope(tie, one, zero, to_bf16=True), np.ones_like(tie))
    tie3 = np.full((1, 1, 1, 2), 1.0 + 3 * 2.0 ** -8, np.float32)   # halfway between 1 + 2^-7 and 1 + 2^-6
    np.testing.assert_array_equal(oracle.rope(tie3, one, zero, to_bf16=True), np.full_like(tie, 1.0 + 2.0 ** -6))


def test_rope_backward_is_the_adjoint():
    L, d = 21, 8
    x, g = _x((1, 2, L, d), 6).astype(np.float64), _x((1, 2, L, d), 7).astype(np.float64)
    cos, sin = rope_tables(L, d)
    # <R x, g> == <x, R^T g> with R applied in float64 here (complex form)
    z = (x[..., 0::2] + 1j * x[..., 1::2]) * (cos.astype(np.float64) + 1j * sin.astype(np.float64))
    Rx = np.empty_like(x)
    Rx[..., 0::2], Rx[..., 1::2] = z.real, z.imag
    lhs = float(np.sum(Rx * g))
    rhs = float(np.sum(x * oracle.rope_bwd(g, cos, sin)))
    assert abs(lhs - rhs) <= 1e-12 * (abs(lhs) + 1.0)
    # and R^T R = identity on the gradient
    back = oracle.rope_bwd(Rx, cos, sin)
    assert np.max(np.abs(back - x)) <= 1e-6   # tables are float32 values: cos^2 + sin^2 = 1 to 1e-7
