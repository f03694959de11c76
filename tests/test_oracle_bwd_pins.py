"""Pins for the backward oracle: central finite differences of the forward oracle with the index decisions frozen,
the dense special case, and closed forms.  CPU only."""
import numpy as np
import pytest

from oracle import isa_oracle as O
from oracle import isa_oracle_bwd as B


def rand_case(rng, seg_len, D, qscale=1.0):
    S = sum(seg_len)
    return rng.standard_normal((S, D)) * qscale, rng.standard_normal((S, D)), rng.standard_normal((S, D))


def directional_fd(f, X, U, eps):
    """<dO, d f(X + t U)/dt> at t = 0 by a fourth-order central difference; f returns <dO, out>."""
    return (-f(X + 2 * eps * U) + 8 * f(X + eps * U) - 8 * f(X - eps * U) + f(X - 2 * eps * U)) / (12 * eps)


def test_dense_backward_matches_finite_differences():
    rng = np.random.default_rng(1)
    Q, K, V = rng.standard_normal((7, 5)), rng.standard_normal((11, 5)), rng.standard_normal((11, 4))
    dO = rng.standard_normal((7, 4))
    dQ, dK, dV = B.dense_attention_bwd(Q, K, V, dO)
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(4):
            U = rng.standard_normal(X.shape)
            f = lambda Y: float((dO * O.dense_attention(*(Y if n == name else Z for n, Z in (("Q", Q), ("K", K), ("V", V))))).sum())
            np.testing.assert_allclose((G * U).sum(), directional_fd(f, X, U, 1e-3), rtol=1e-7, atol=1e-9)


def test_dense_backward_closed_forms():
    rng = np.random.default_rng(2)
    # one key: the output is that key's value whatever q is -> dQ = dK = 0, dV = column sums of dO
    Q, K, V, dO = rng.standard_normal((5, 3)), rng.standard_normal((1, 3)), rng.standard_normal((1, 2)), rng.standard_normal((5, 2))
    dQ, dK, dV = B.dense_attention_bwd(Q, K, V, dO)
    np.testing.assert_allclose(dQ, 0, atol=1e-15)
    np.testing.assert_allclose(dK, 0, atol=1e-15)
    np.testing.assert_allclose(dV, dO.sum(axis=0, keepdims=True), atol=1e-14)
    # zero queries: uniform weights 1/n -> dV_t = mean-of-rows share, every row of dV = sum_i dO_i / n
    Q, K, V, dO = np.zeros((4, 3)), rng.standard_normal((6, 3)), rng.standard_normal((6, 2)), rng.standard_normal((4, 2))
    _, _, dV = B.dense_attention_bwd(Q, K, V, dO)
    np.testing.assert_allclose(dV, np.tile(dO.sum(axis=0) / 6, (6, 1)), atol=1e-14)


@pytest.mark.parametrize("seed,gamma,exact_frac", [(0, 0.0, 0.0), (1, 0.0, 0.3), (2, 0.6, 0.0), (3, -0.4, 0.25), (4, 0.0, 1.0)])
def test_isa_backward_matches_finite_differences(seed, gamma, exact_frac):
    rng = np.random.default_rng(40 + seed)
    b = [2, 3, 4, 4, 3][seed]
    seg = [int(rng.integers(9, 16)), int(rng.integers(5, 12))] + ([int(rng.integers(2, 6))] if seed % 2 else [])
    Q, K, V = rand_case(rng, seg, int(rng.integers(3, 6)), qscale=1.5)
    dO = rng.standard_normal(V.shape)
    out, plan = O.isa_attention(Q, K, V, seg, b, 0.5, 0.4, exact_frac, gamma=gamma)
    # the frozen-index forward reproduces the operator at the expansion point
    np.testing.assert_allclose(B.forward_with_fixed_indices(Q, K, V, plan), out, rtol=0, atol=1e-13)
    dQ, dK, dV = B.isa_attention_bwd(Q, K, V, dO, plan)
    tensors = {"Q": Q, "K": K, "V": V}
    for name, G in (("Q", dQ), ("K", dK), ("V", dV)):
        for _ in range(3):
            U = rng.standard_normal(tensors[name].shape)
            def f(Y):
                args = dict(tensors)
                args[name] = Y
                return float((dO * B.forward_with_fixed_indices(args["Q"], args["K"], args["V"], plan)).sum())
            np.testing.assert_allclose((G * U).sum(), directional_fd(f, tensors[name], U, 1e-3), rtol=2e-7, atol=1e-9)


def test_isa_backward_reduces_to_dense_backward():
    rng = np.random.default_rng(9)
    seg = [13, 10]
    Q, K, V = rand_case(rng, seg, 4)
    dO = rng.standard_normal(V.shape)
    _, plan = O.isa_attention(Q, K, V, seg, 4, 1.0, 1.0)                 # everything kept, everything exact
    got = B.isa_attention_bwd(Q, K, V, dO, plan)
    want = B.dense_attention_bwd(Q, K, V, dO)
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, rtol=0, atol=1e-13)


def test_unused_context_blocks_get_no_gradient():
    rng = np.random.default_rng(10)
    seg = [16, 16]
    Q, K, V = rand_case(rng, seg, 4)
    dO = rng.standard_normal(V.shape)
    _, plan = O.isa_attention(Q, K, V, seg, 4, 0.5, 0.5, 0.25)
    _, dK, dV = B.isa_attention_bwd(Q, K, V, dO, plan)
    dropped = [j for j in range(plan["T"]) if j not in set(plan["kv_list"].tolist())]
    assert dropped
    for j in dropped:
        rows = slice(plan["starts"][j], plan["starts"][j] + plan["counts"][j])
        assert not dK[rows].any() and not dV[rows].any()                   # pruned keys never enter the forward
    # the gradients of V sum to the column sums of dO: every output row is a convex combination of values
    np.testing.assert_allclose(dV.sum(axis=0), dO.sum(axis=0), atol=1e-12)


def test_taylor_mean_gradient_is_shared_evenly_inside_a_block():
    rng = np.random.default_rng(11)
    seg = [12, 8]
    Q, K, V = rand_case(rng, seg, 4)
    dO = rng.standard_normal(V.shape)
    _, plan = O.isa_attention(Q, K, V, seg, 4, 1.0, 0.0)                   # every block Taylor, no exact sets
    _, dK, dV = B.isa_attention_bwd(Q, K, V, dO, plan)
    for j in range(plan["T"]):
        rows = slice(plan["starts"][j], plan["starts"][j] + plan["counts"][j])
        np.testing.assert_allclose(dK[rows], np.tile(dK[rows][:1], (plan["counts"][j], 1)), atol=1e-14)
        np.testing.assert_allclose(dV[rows], np.tile(dV[rows][:1], (plan["counts"][j], 1)), atol=1e-14)


def test_restriction_to_query_blocks_is_the_gradient_for_a_masked_dO():
    """The query_blocks argument only drops terms of the sum over query blocks: same result as zeroing dO elsewhere."""
    rng = np.random.default_rng(11)
    seg, block, D = [70, 45], 16, 8
    S = sum(seg)
    Q, K, V, dO = (rng.standard_normal((S, D)) for _ in range(4))
    plan = O.isa_plan(Q, K, V, seg, block, 0.5, 0.4, 0.0, 0.0)
    pick = [int(plan["full_list"][0]), int(plan["flat_list"][-1])]
    masked = np.zeros_like(dO)
    for i in pick:
        rows = slice(plan["starts"][i], plan["starts"][i] + plan["counts"][i])
        masked[rows] = dO[rows]
    a = B.isa_attention_bwd(Q, K, V, dO, plan, query_blocks=pick)
    b = B.isa_attention_bwd(Q, K, V, masked, plan)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=0, atol=1e-13)
