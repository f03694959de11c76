"""fp64 CPU oracle of the backward pass of In-Context Sparse Attention (ISA).

TEST INFRASTRUCTURE ONLY, like isa_oracle.py, whose forward definitions it
differentiates.  The paper states that a backward pass exists (Sec. 4
"Implementation Detail and Analysis") and gives no formulas for it, so the
oracle is the analytic gradient of the forward operator as isa_oracle.py
defines it, with every index decision of Alg. 1 (kept context blocks, query
groups, exact sets) held fixed: those are piecewise constant in the inputs.
Everything else is differentiated, including the block means that feed the
Taylor branch (Eq. 4) and the coarse residual gamma * O_coarse (Alg. 1
Stages 1 and 5).

Pinned by central finite differences of the forward oracle with the same
indices frozen, by the dense special case, and by closed forms
(tests/test_oracle_bwd_pins.py).
"""
import math

import numpy as np

from . import isa_oracle as O


def dense_attention_bwd(Q, K, V, dO):
    """Gradients of dense_attention: (dQ, dK, dV) for O = softmax(Q K^T / sqrt(D)) V."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    scale = 1.0 / math.sqrt(Q.shape[1])
    s = (Q @ K.T) * scale
    p = np.exp(s - s.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    o = p @ V
    delta = (dO * o).sum(axis=1, keepdims=True)
    dS = p * (dO @ V.T - delta)
    return dS @ K * scale, dS.T @ Q * scale, p.T @ dO


def forward_with_fixed_indices(Q, K, V, plan):
    """Alg. 1 with the index lists (and exact sets) of `plan` held fixed while block means, coarse map and coarse
    output follow the given Q, K, V.  This is the function whose gradient isa_attention_bwd returns."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    starts, counts = plan["starts"], plan["counts"]
    fresh = dict(plan)
    fresh["Qc"] = O.block_means(Q, starts, counts)
    fresh["Kc"] = O.block_means(K, starts, counts)
    fresh["Vc"] = O.block_means(V, starts, counts)
    fresh["O_coarse"] = O.coarse_output(O.coarse_map(O.coarse_logits(fresh["Qc"], fresh["Kc"])), fresh["Vc"])
    out = np.zeros((Q.shape[0], V.shape[1]))
    full = set(int(i) for i in plan["full_list"])
    for i in range(plan["T"]):
        ex = None if i in full else exact_blocks_of(plan, i)
        out[starts[i]:starts[i] + counts[i]] = O.attend_block(i, fresh, Q, K, V, kv_list=plan["kv_list"],
                                                              in_full=i in full, exact_blocks=ex)
    return out


def exact_blocks_of(plan, i):
    """The exact set E_i of Taylor query block i under the plan's own pooled logits (Alg. 2 Part A selection)."""
    return O.exact_set(plan["Z"][i], plan["kv_list"], O.exact_count(plan["exact_frac"], len(plan["kv_list"])))


def isa_attention_bwd(Q, K, V, dO, plan, query_blocks=None):
    """Gradient of forward_with_fixed_indices with respect to Q, K, V, contracted with dO.  Returns (dQ, dK, dV).
    `query_blocks` restricts the sum to the given query blocks (the gradient is a sum of per-query-block terms): the
    result is then the gradient for a dO that is zero on all other blocks, whatever dO holds there."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    starts, counts, T = plan["starts"], plan["counts"], plan["T"]
    D = Q.shape[1]
    scale = 1.0 / math.sqrt(D)
    kv_list = np.asarray(plan["kv_list"], dtype=np.int64)
    full = set(int(i) for i in plan["full_list"])
    gamma = plan["gamma"]
    Qc, Kc, Vc = (O.block_means(X, starts, counts) for X in (Q, K, V))
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    dQc, dKc, dVc = np.zeros_like(Qc), np.zeros_like(Kc), np.zeros_like(Vc)
    dOc = np.zeros_like(Vc)

    def tokens_of(blocks):
        if len(blocks) == 0:
            return np.zeros(0, dtype=np.int64)
        return np.concatenate([np.arange(starts[j], starts[j] + counts[j]) for j in blocks])

    for i in (range(T) if query_blocks is None else query_blocks):
        rows = slice(starts[i], starts[i] + counts[i])
        q, do = Q[rows], dO[rows]
        if gamma != 0.0:
            dOc[i] = gamma * do.sum(axis=0)                       # the block's coarse row is shared by its tokens
        if i in full:
            exact, mean_blocks = kv_list, np.zeros(0, dtype=np.int64)
        else:
            exact = np.asarray(exact_blocks_of(plan, i), dtype=np.int64)
            mean_blocks = np.asarray([j for j in kv_list if j not in set(exact.tolist())], dtype=np.int64)
        tok = tokens_of(exact)
        s_e = (q @ K[tok].T) * scale
        s_m = (q @ Kc[mean_blocks].T) * scale
        m = np.full((q.shape[0], 1), -np.inf)
        if s_e.shape[1]:
            m = np.maximum(m, s_e.max(axis=1, keepdims=True))
        if s_m.shape[1]:
            m = np.maximum(m, s_m.max(axis=1, keepdims=True))
        a_e = np.exp(s_e - m)
        a_m = np.exp(s_m - m) * counts[mean_blocks].astype(np.float64)[None, :]     # Eq. 4: a mean key weighs n_j
        ell = a_e.sum(axis=1, keepdims=True) + a_m.sum(axis=1, keepdims=True)
        a_e, a_m = a_e / ell, a_m / ell
        o = a_e @ V[tok] + a_m @ Vc[mean_blocks]
        delta = (do * o).sum(axis=1, keepdims=True)
        dS_e = a_e * (do @ V[tok].T - delta)
        dS_m = a_m * (do @ Vc[mean_blocks].T - delta)
        dQ[rows] += (dS_e @ K[tok] + dS_m @ Kc[mean_blocks]) * scale
        np.add.at(dK, tok, dS_e.T @ q * scale)
        np.add.at(dV, tok, a_e.T @ do)
        np.add.at(dKc, mean_blocks, dS_m.T @ q * scale)
        np.add.at(dVc, mean_blocks, a_m.T @ do)

    if gamma != 0.0:                                              # O_coarse = softmax(Qc Kc^T / sqrt(D)) Vc
        S = O.coarse_map(O.coarse_logits(Qc, Kc))
        dVc += S.T @ dOc
        dS = dOc @ Vc.T
        dZ = S * (dS - (dS * S).sum(axis=1, keepdims=True))
        dQc += dZ @ Kc * scale
        dKc += dZ.T @ Qc * scale

    for j in range(T):                                            # a block mean spreads its gradient evenly over its tokens
        rows = slice(starts[j], starts[j] + counts[j])
        dQ[rows] += dQc[j] / counts[j]
        dK[rows] += dKc[j] / counts[j]
        dV[rows] += dVc[j] / counts[j]
    return dQ, dK, dV
