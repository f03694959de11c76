"""Pins for the fp64 oracle: every check compares it with something other than
itself -- a naive long-double evaluator written separately below, closed forms,
invariants of the definitions, scipy routines in special cases, and the few
numbers the paper prints.  None of these tests needs a GPU."""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import isa_oracle as O

LD = np.longdouble


# --------------------------------------------------------------------------
# A separate, naive evaluator: scalar loops, long double, no max subtraction,
# rankings by sorting (value, index) tuples.  Tiny inputs only.
# --------------------------------------------------------------------------
def brute_isa(Q, K, V, seg_len, b, keep_ratio, full_frac, exact_frac):
    S_tot, D = Q.shape
    blk_of = []
    blocks = []                                   # token lists
    for si, L in enumerate(seg_len):
        base = sum(seg_len[:si])
        nb = (L + b - 1) // b
        for x in range(nb):
            blocks.append([base + t for t in range(x * b, min(L, (x + 1) * b))])
    for j, toks in enumerate(blocks):
        for _ in toks:
            blk_of.append(j)
    T = len(blocks)
    T_src = (seg_len[0] + b - 1) // b

    def mean_of(X, toks):
        acc = [LD(0)] * D
        for t in toks:
            for d in range(D):
                acc[d] += LD(X[t, d])
        return [a / LD(len(toks)) for a in acc]

    Qc = [mean_of(Q, tk) for tk in blocks]
    Kc = [mean_of(K, tk) for tk in blocks]
    Vc = [mean_of(V, tk) for tk in blocks]
    rD = LD(1) / np.sqrt(LD(D))
    Z = [[sum(Qc[i][d] * Kc[j][d] for d in range(D)) * rD for j in range(T)] for i in range(T)]
    Sc = []
    for i in range(T):
        e = [np.exp(z) for z in Z[i]]
        tot = sum(e)
        Sc.append([x / tot for x in e])
    T_ctx = T - T_src
    s_ctx = [sum(Sc[i][T_src + j] for i in range(T_src)) / LD(T_src) for j in range(T_ctx)]
    k_keep = int(math.floor(keep_ratio * T_ctx))
    ranked = sorted(range(T_ctx), key=lambda j: (-s_ctx[j], j))
    kv = list(range(T_src)) + sorted(T_src + j for j in ranked[:k_keep])
    sharp = []
    for i in range(T):
        mu = sum(Sc[i][:T_src]) / LD(T_src)
        sharp.append(sum((x - mu) ** 2 for x in Sc[i][:T_src]) / LD(T_src))
    n_flat = int(math.floor((1.0 - full_frac) * T))
    n_full = T - n_flat
    order = sorted(range(T), key=lambda i: (-sharp[i], i))
    full = set(order[:n_full])
    k_exact = int(math.floor(exact_frac * len(kv)))

    out = np.zeros((S_tot, D))
    for tq in range(S_tot):
        i = blk_of[tq]
        q = [LD(x) for x in Q[tq]]
        num = [LD(0)] * D
        den = LD(0)
        if i in full:
            exact = kv
        else:
            pos = sorted(range(len(kv)), key=lambda p: (-Z[i][kv[p]], p))[:k_exact]
            exact = [kv[p] for p in pos]
        for j in kv:
            if j in exact:
                for t in blocks[j]:
                    w = np.exp(sum(q[d] * LD(K[t, d]) for d in range(D)) * rD)
                    den += w
                    for d in range(D):
                        num[d] += w * LD(V[t, d])
            else:
                w = np.exp(sum(q[d] * Kc[j][d] for d in range(D)) * rD) * LD(len(blocks[j]))
                den += w
                for d in range(D):
                    num[d] += w * Vc[j][d]
        out[tq] = [float(x / den) for x in num]
    return out, dict(kv=kv, full=sorted(full), s_ctx=[float(x) for x in s_ctx], sharp=[float(x) for x in sharp])


def rand_case(rng, seg_len, D, qscale=1.0):
    S = sum(seg_len)
    Q = rng.standard_normal((S, D)) * qscale
    K = rng.standard_normal((S, D))
    V = rng.standard_normal((S, D))
    return Q, K, V


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_tiny(seed):
    rng = np.random.default_rng(100 + seed)
    b = [1, 2, 4, 8][seed % 4]
    seg_len = [int(rng.integers(5, 15)), int(rng.integers(3, 12))]
    if seed % 3 == 0:
        seg_len.append(int(rng.integers(1, 7)))            # a second context reference
    D = int(rng.integers(2, 7))
    keep, full, exact = float(rng.uniform(0, 1)), float(rng.uniform(0, 1)), float(rng.uniform(0, 0.6))
    Q, K, V = rand_case(rng, seg_len, D, qscale=2.0)
    want, info = brute_isa(Q, K, V, seg_len, b, keep, full, exact)
    got, plan = O.isa_attention(Q, K, V, seg_len, b, keep, full, exact)
    assert list(plan["kv_list"]) == info["kv"]
    assert list(plan["full_list"]) == info["full"]
    np.testing.assert_allclose(plan["s_ctx"], info["s_ctx"], rtol=1e-12, atol=0)
    np.testing.assert_allclose(plan["sharp"], info["sharp"], rtol=1e-10, atol=1e-300)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# Dense attention against a library softmax and a scalar evaluation
# --------------------------------------------------------------------------
def test_dense_matches_scipy_softmax():
    rng = np.random.default_rng(1)
    Q, K, V = rng.standard_normal((7, 5)) * 3, rng.standard_normal((11, 5)), rng.standard_normal((11, 3))
    want = scipy.special.softmax(Q @ K.T / math.sqrt(5), axis=1) @ V
    np.testing.assert_allclose(O.dense_attention(Q, K, V), want, rtol=0, atol=1e-13)


def test_dense_single_key_and_uniform():
    rng = np.random.default_rng(2)
    V = rng.standard_normal((6, 4))
    Q = rng.standard_normal((3, 4))
    # one key: the output is that key's value whatever the logits are
    np.testing.assert_allclose(O.dense_attention(Q, Q[:1] * 50, V[:1]), np.repeat(V[:1], 3, 0), atol=1e-15)
    # zero queries: uniform weights, output = plain mean of V
    np.testing.assert_allclose(O.dense_attention(Q * 0, rng.standard_normal((6, 4)), V),
                               np.repeat(V.mean(0, keepdims=True), 3, 0), atol=1e-15)


def test_dense_large_logits_stay_finite():
    Q = np.full((2, 4), 200.0)
    K = np.vstack([np.full((1, 4), 200.0), np.zeros((3, 4))])
    V = np.arange(16.0).reshape(4, 4)
    out = O.dense_attention(Q, K, V)
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out, np.repeat(V[:1], 2, 0), atol=1e-12)


# --------------------------------------------------------------------------
# Block layout, counts, and the numbers the paper prints
# --------------------------------------------------------------------------
def test_block_layout_segment_aligned():
    starts, counts, T_src = O.block_layout([10, 3, 9], 4)
    assert T_src == 3
    assert list(starts) == [0, 4, 8, 10, 13, 17, 21]
    assert list(counts) == [4, 4, 2, 3, 4, 4, 1]
    assert counts.sum() == 22


def test_block_means_by_hand():
    X = np.array([[1.0, 10.0], [3.0, 30.0], [5.0, 50.0], [7.0, 70.0], [100.0, -100.0]])
    starts, counts, _ = O.block_layout([5], 2)
    np.testing.assert_array_equal(O.block_means(X, starts, counts),
                                  np.array([[2.0, 20.0], [6.0, 60.0], [100.0, -100.0]]))


def _paper_values():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                vals[line[0]] = float(line[1])
    return vals


def test_counts_match_paper_numbers():
    pv = _paper_values()
    # Sec. 3: with the default No-Sparsity Ratio the Taylor component skips 93.75 % of the blocks.
    for T_new in (16, 384, 512, 1184):
        k = O.exact_count(pv["default_alpha_ns"], T_new)
        assert 1.0 - k / T_new == pytest.approx(pv["taylor_sparsity_at_default_alpha_ns"], abs=1e-12)
    # Sec. 3 complexity claim: with divisible lengths K_new holds L_src + alpha_s * L_ctx tokens.
    b, L_src, L_ctx = 8, 64, 128
    starts, counts, T_src = O.block_layout([L_src, L_ctx], b)
    kv = O.preselect(np.arange(L_ctx // b, dtype=float), O.keep_count(pv["default_alpha_s"], L_ctx // b), T_src)
    assert counts[kv].sum() == L_src + pv["default_alpha_s"] * L_ctx
    # Alg. 1 Stage 3 split with alpha_f(alg) = 1 - full_frac, on the block counts of the benchmark shapes
    assert O.group_counts(0.25, 16) == (4, 12)
    assert O.group_counts(0.25, 122) == (31, 91)
    assert O.group_counts(0.2, 512) == (103, 409)
    assert O.group_counts(0.2, 1182) == (237, 945)
    assert O.group_counts(pv["default_alpha_f"], 512) == (256, 256)
    assert O.keep_count(0.5, 61) == 30 and O.keep_count(0.5, 256) == 128 and O.keep_count(0.5, 591) == 295
    assert O.keep_count(0.0, 9) == 0 and O.keep_count(1.0, 9) == 9


def test_rankings_ties_and_order():
    assert list(O.top_indices([1.0, 3.0, 3.0, 2.0, 3.0], 3)) == [1, 2, 4]          # ties -> lower index
    assert list(O.top_indices([1.0, 3.0, 3.0, 2.0, 3.0], 4)) == [1, 2, 4, 3]
    kv = O.preselect(np.array([0.1, 0.9, 0.5, 0.9]), 2, 3)
    assert list(kv) == [0, 1, 2, 3 + 1, 3 + 3]
    full, flat = O.group_queries(np.array([0.0, 5.0, 1.0, 5.0, 2.0]), 2)
    assert list(full) == [1, 3] and list(flat) == [0, 2, 4]
    assert list(O.exact_set(np.array([9.0, 1.0, 7.0, 7.0, 8.0]), np.array([1, 2, 3, 4]), 2)) == [2, 4]


# --------------------------------------------------------------------------
# Closed forms for the coarse map, the saliency and the sharpness
# --------------------------------------------------------------------------
def test_uniform_coarse_map_closed_form():
    rng = np.random.default_rng(3)
    seg = [12, 9]
    Q, K, V = rand_case(rng, seg, 4)
    _, plan = O.isa_attention(Q * 0, K, V, seg, 4, 0.5, 0.5)
    T = plan["T"]
    np.testing.assert_allclose(plan["S_coarse"], np.full((T, T), 1.0 / T), atol=1e-16)
    np.testing.assert_allclose(plan["s_ctx"], 1.0 / T, atol=1e-16)
    np.testing.assert_allclose(plan["sharp"], 0.0, atol=1e-30)
    # all tied: ties go to the lower index
    assert list(plan["kv_list"]) == [0, 1, 2, 3]
    assert list(plan["full_list"]) == [0, 1, 2]


def test_one_hot_rows_closed_form():
    # Query block i looks (with a huge logit) at key block c(i): S_coarse rows are one-hot.
    T_src, T_ctx, D = 4, 3, 8
    T = T_src + T_ctx
    Kc = np.eye(T, D) * 40.0                       # key block j = 40 e_j  (T <= D)
    target = [2, 0, 5, 1, 6, 6, 3]                 # column each query block looks at
    Qc = np.stack([Kc[c] for c in target])
    S = O.coarse_map(O.coarse_logits(Qc, Kc))
    M = O.sharpness(S, T_src)
    for i, c in enumerate(target):
        want = (1.0 / T_src) * (1.0 - 1.0 / T_src) if c < T_src else 0.0
        assert M[i] == pytest.approx(want, abs=1e-12)
    # saliency: source query blocks 0..3 look at columns 2, 0, 5, 1 -> only context block 5 gets 1/T_src
    np.testing.assert_allclose(O.context_saliency(S, T_src), [0.0, 0.25, 0.0], atol=1e-12)


def test_scaled_softmax_uses_sqrt_d():
    # two key blocks, logits differ by exactly ln(3) after the 1/sqrt(D) scaling -> weights 3/4, 1/4
    D = 16
    Qc = np.zeros((1, D)); Qc[0, 0] = 4.0
    Kc = np.zeros((2, D)); Kc[0, 0] = math.log(3.0)
    S = O.coarse_map(O.coarse_logits(Qc, Kc))
    np.testing.assert_allclose(S, [[0.75, 0.25]], atol=1e-15)


# --------------------------------------------------------------------------
# Selection direction, checked on a case whose answer is known by construction
# --------------------------------------------------------------------------
def _planted_case(rng, b=4, D=6):
    """Source queries share a +e0 component; context blocks 1 and 4 (of 6) carry keys along +e0,
    the others along -e0, so blocks 1 and 4 are the two most salient."""
    seg = [5 * b + 1, 6 * b - 2]                   # short tails on both segments
    S = sum(seg)
    Q = 0.1 * rng.standard_normal((S, D)); Q[:, 0] += 3.0
    K = 0.1 * rng.standard_normal((S, D))
    V = rng.standard_normal((S, D))
    starts, counts, T_src = O.block_layout(seg, b)
    for j in range(T_src, len(starts)):
        sign = 1.0 if (j - T_src) in (1, 4) else -1.0
        K[starts[j]:starts[j] + counts[j], 0] += 2.0 * sign
    return seg, Q, K, V, starts, counts, T_src


def test_preselection_only_equals_dense_on_planted_blocks():
    rng = np.random.default_rng(4)
    b = 4
    seg, Q, K, V, starts, counts, T_src = _planted_case(rng, b)
    out, plan = O.isa_attention(Q, K, V, seg, b, keep_ratio=2 / 6 + 1e-9, full_frac=1.0)
    assert plan["k_keep"] == 2
    assert list(plan["kv_list"][T_src:]) == [T_src + 1, T_src + 4]
    tok = list(range(seg[0]))
    for j in (T_src + 1, T_src + 4):
        tok += list(range(starts[j], starts[j] + counts[j]))
    want = scipy.special.softmax(Q @ K[tok].T / math.sqrt(Q.shape[1]), axis=1) @ V[tok]
    np.testing.assert_allclose(out, want, atol=1e-13)


def test_grouping_sends_sharp_blocks_to_exact_branch():
    # query blocks 1 and 3 have large norm along one source key block's mean -> peaked coarse rows
    rng = np.random.default_rng(5)
    b, D = 4, 8
    seg = [16, 8]
    S = sum(seg)
    K = 0.05 * rng.standard_normal((S, D))
    K[0:4, 1] += 3.0                                # source key block 0 points along e1
    Q = 0.05 * rng.standard_normal((S, D))
    Q[4:8, 1] += 6.0                                # query block 1: sharp
    Q[12:16, 1] += 5.0                              # query block 3: sharp
    V = rng.standard_normal((S, D))
    out, plan = O.isa_attention(Q, K, V, seg, b, keep_ratio=1.0, full_frac=0.3)
    assert plan["n_full"] == 2
    assert list(plan["full_list"]) == [1, 3]
    assert sorted(list(plan["full_list"]) + list(plan["flat_list"])) == list(range(6))
    # rows of the exact group equal dense attention, rows of the Taylor group do not
    dense = O.dense_attention(Q, K, V)
    np.testing.assert_allclose(out[4:8], dense[4:8], atol=1e-13)
    np.testing.assert_allclose(out[12:16], dense[12:16], atol=1e-13)
    assert np.abs(out[0:4] - dense[0:4]).max() > 1e-6


# --------------------------------------------------------------------------
# Invariants of the definitions
# --------------------------------------------------------------------------
SEGS = [[21, 13], [16, 16], [9, 5, 11]]


@pytest.mark.parametrize("seg", SEGS)
def test_isa_equals_dense_when_everything_is_exact(seg):
    rng = np.random.default_rng(6)
    Q, K, V = rand_case(rng, seg, 5, qscale=2.0)
    out, plan = O.isa_attention(Q, K, V, seg, 4, keep_ratio=1.0, full_frac=1.0)
    assert plan["n_flat"] == 0 and len(plan["kv_list"]) == plan["T"]
    np.testing.assert_allclose(out, O.dense_attention(Q, K, V), atol=1e-13)


@pytest.mark.parametrize("seg", SEGS)
def test_taylor_exact_when_keys_in_a_block_coincide(seg):
    """Eq. 4 is exact when every key of a block equals the block mean, for any values, and
    only with the real token count n_j as weight for a short tail block."""
    rng = np.random.default_rng(7)
    b = 4
    Q, K, V = rand_case(rng, seg, 5, qscale=2.0)
    starts, counts, _ = O.block_layout(seg, b)
    for s, n in zip(starts, counts):
        K[s:s + n] = K[s]
    out, plan = O.isa_attention(Q, K, V, seg, b, keep_ratio=1.0, full_frac=0.0)
    assert plan["n_full"] == 0
    np.testing.assert_allclose(out, O.dense_attention(Q, K, V), atol=1e-13)


def test_taylor_exact_at_block_size_one():
    rng = np.random.default_rng(8)
    seg = [11, 7]
    Q, K, V = rand_case(rng, seg, 4, qscale=2.0)
    out, _ = O.isa_attention(Q, K, V, seg, 1, keep_ratio=1.0, full_frac=0.0)
    np.testing.assert_allclose(out, O.dense_attention(Q, K, V), atol=1e-13)


@pytest.mark.parametrize("seg", SEGS)
def test_exact_frac_one_is_exact_attention_over_kept_keys(seg):
    rng = np.random.default_rng(9)
    Q, K, V = rand_case(rng, seg, 5, qscale=2.0)
    a, pa = O.isa_attention(Q, K, V, seg, 4, keep_ratio=0.5, full_frac=0.0, exact_frac=1.0)
    f, pf = O.isa_attention(Q, K, V, seg, 4, keep_ratio=0.5, full_frac=1.0)
    assert list(pa["kv_list"]) == list(pf["kv_list"])
    np.testing.assert_allclose(a, f, atol=1e-13)


@pytest.mark.parametrize("seg", SEGS)
@pytest.mark.parametrize("ratios", [(0.5, 0.3, 0.0), (0.0, 0.0, 0.25), (0.7, 0.6, 0.5)])
def test_constant_values_give_constant_output(seg, ratios):
    """With V == 1 every output is 1: the n_j weights must enter numerator and normaliser alike."""
    rng = np.random.default_rng(10)
    Q, K, V = rand_case(rng, seg, 5, qscale=2.0)
    out, _ = O.isa_attention(Q, K, np.ones_like(V), seg, 4, *ratios)
    np.testing.assert_allclose(out, 1.0, atol=1e-14)


@pytest.mark.parametrize("seg", SEGS)
def test_zero_queries_give_mean_of_kept_values(seg):
    """q = 0: uniform weights.  Exact branch -> mean of V over kept tokens; Taylor branch ->
    sum_j n_j V^c_j / sum_j n_j, which is the same number."""
    rng = np.random.default_rng(11)
    Q, K, V = rand_case(rng, seg, 5)
    out, plan = O.isa_attention(Q * 0, K, V, seg, 4, keep_ratio=0.5, full_frac=0.4, exact_frac=0.3)
    tok = np.concatenate([np.arange(plan["starts"][j], plan["starts"][j] + plan["counts"][j])
                          for j in plan["kv_list"]])
    np.testing.assert_allclose(out, np.repeat(V[tok].mean(0, keepdims=True), len(Q), 0), atol=1e-14)


@pytest.mark.parametrize("seg", SEGS)
def test_key_shift_invariance(seg):
    rng = np.random.default_rng(12)
    Q, K, V = rand_case(rng, seg, 5, qscale=1.5)
    c = rng.standard_normal((1, 5))
    a, pa = O.isa_attention(Q, K, V, seg, 4, 0.5, 0.3, 0.25)
    s, ps = O.isa_attention(Q, K + c, V, seg, 4, 0.5, 0.3, 0.25)
    np.testing.assert_allclose(ps["S_coarse"], pa["S_coarse"], atol=1e-14)
    assert list(ps["kv_list"]) == list(pa["kv_list"]) and list(ps["full_list"]) == list(pa["full_list"])
    np.testing.assert_allclose(s, a, atol=1e-12)


def test_jensen_taylor_normaliser_is_a_lower_bound():
    rng = np.random.default_rng(13)
    seg = [22, 15]
    Q, K, V = rand_case(rng, seg, 6, qscale=2.0)
    plan = O.isa_plan(Q, K, V, seg, 4, 0.6, 0.0)
    kv = plan["kv_list"]
    args = (Q, K, V, plan["Kc"], plan["Vc"], plan["starts"], plan["counts"], kv)
    _, ell_t, m_t = O.taylor_branch(*args, exact_blocks=[], return_parts=True)
    _, ell_e, m_e = O.taylor_branch(*args, exact_blocks=list(kv), return_parts=True)
    log_t = np.log(ell_t) + m_t
    log_e = np.log(ell_e) + m_e
    assert np.all(log_t <= log_e + 1e-12)
    assert np.any(log_t < log_e - 1e-6)


def test_kv_list_order_does_not_matter():
    rng = np.random.default_rng(14)
    seg = [19, 14]
    Q, K, V = rand_case(rng, seg, 5, qscale=2.0)
    plan = O.isa_plan(Q, K, V, seg, 4, 0.5, 0.5, 0.25)
    perm = rng.permutation(len(plan["kv_list"]))
    for i in (int(plan["full_list"][0]), int(plan["flat_list"][0])):
        ex = O.exact_set(plan["Z"][i], plan["kv_list"], plan["k_exact"])
        a = O.attend_block(i, plan, Q, K, V, exact_blocks=ex)
        bb = O.attend_block(i, plan, Q, K, V, kv_list=plan["kv_list"][perm], exact_blocks=ex)
        np.testing.assert_allclose(a, bb, atol=1e-12)


@pytest.mark.parametrize("seed", range(5))
def test_lists_partition_and_are_sorted(seed):
    rng = np.random.default_rng(20 + seed)
    seg = [int(rng.integers(4, 40)), int(rng.integers(1, 40)), int(rng.integers(1, 20))]
    Q, K, V = rand_case(rng, seg, 4)
    plan = O.isa_plan(Q, K, V, seg, 4, float(rng.uniform()), float(rng.uniform()))
    T, T_src = plan["T"], plan["T_src"]
    assert plan["n_full"] + plan["n_flat"] == T
    assert sorted(list(plan["full_list"]) + list(plan["flat_list"])) == list(range(T))
    kv = list(plan["kv_list"])
    assert kv[:T_src] == list(range(T_src)) and all(x < y for x, y in zip(kv, kv[1:]))
    assert len(kv) == T_src + plan["k_keep"] and max(kv) < T


def test_taylor_error_is_second_order_in_the_spread():
    """Expanding around the block MEAN cancels the first-order term, so halving the spread of
    keys and values inside blocks must quarter the error."""
    rng = np.random.default_rng(15)
    seg, b, D = [32, 16], 8, 6
    S = sum(seg)
    starts, counts, _ = O.block_layout(seg, b)
    base_k = np.repeat(rng.standard_normal((len(starts), D)), counts, axis=0)
    base_v = np.repeat(rng.standard_normal((len(starts), D)), counts, axis=0)
    dk, dv = rng.standard_normal((S, D)), rng.standard_normal((S, D))
    Q = rng.standard_normal((S, D))

    def err(eps):
        K, V = base_k + eps * dk, base_v + eps * dv
        out, _ = O.isa_attention(Q, K, V, seg, b, 1.0, 0.0)
        return np.abs(out - O.dense_attention(Q, K, V)).max()

    e1, e2 = err(1e-2), err(5e-3)
    assert 3.6 < e1 / e2 < 4.4


# --------------------------------------------------------------------------
# Coarse residual gamma * O_coarse (Alg. 1 Stage 1 and Stage 5)
# --------------------------------------------------------------------------
def brute_coarse_output(Q, K, V, seg_len, b):
    """O_coarse from the definitions with scalar long-double loops: block means, pooled logits / sqrt(D), row
    softmax without max subtraction, weighted sum of the mean values."""
    S_tot, D = Q.shape
    blocks = []
    for si, L in enumerate(seg_len):
        base = sum(seg_len[:si])
        for x in range((L + b - 1) // b):
            blocks.append([base + t for t in range(x * b, min(L, (x + 1) * b))])
    T = len(blocks)

    def mean_of(X, toks):
        return [sum(LD(X[t, d]) for t in toks) / LD(len(toks)) for d in range(X.shape[1])]
    Qc = [mean_of(Q, tk) for tk in blocks]
    Kc = [mean_of(K, tk) for tk in blocks]
    Vc = [mean_of(V, tk) for tk in blocks]
    out = np.zeros((T, V.shape[1]), dtype=LD)
    for i in range(T):
        w = [np.exp(sum(Qc[i][d] * Kc[j][d] for d in range(D)) / np.sqrt(LD(D))) for j in range(T)]
        tot = sum(w)
        for d in range(V.shape[1]):
            out[i, d] = sum(w[j] * Vc[j][d] for j in range(T)) / tot
    return out, blocks


@pytest.mark.parametrize("seed", range(4))
def test_coarse_residual_brute_force(seed):
    rng = np.random.default_rng(500 + seed)
    b = [2, 3, 4, 8][seed]
    seg = [int(rng.integers(6, 15)), int(rng.integers(3, 12))]
    Q, K, V = rand_case(rng, seg, int(rng.integers(2, 6)))
    gamma = float(rng.uniform(-1, 1))
    base, _ = O.isa_attention(Q, K, V, seg, b, 0.5, 0.5, 0.25)
    got, plan = O.isa_attention(Q, K, V, seg, b, 0.5, 0.5, 0.25, gamma=gamma)
    oc, blocks = brute_coarse_output(Q, K, V, seg, b)
    np.testing.assert_allclose(plan["O_coarse"], oc.astype(np.float64), rtol=0, atol=1e-13)
    want = base.copy()
    for i, toks in enumerate(blocks):                           # a block's coarse row goes to each of its tokens
        want[toks] += gamma * oc[i].astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_coarse_residual_zero_gamma_changes_nothing_and_is_linear():
    rng = np.random.default_rng(7)
    seg = [19, 14, 6]
    Q, K, V = rand_case(rng, seg, 5)
    o0, _ = O.isa_attention(Q, K, V, seg, 4, 0.4, 0.3, 0.2)
    o0b, _ = O.isa_attention(Q, K, V, seg, 4, 0.4, 0.3, 0.2, gamma=0.0)
    assert np.array_equal(o0, o0b)
    o1, p1 = O.isa_attention(Q, K, V, seg, 4, 0.4, 0.3, 0.2, gamma=1.0)
    o2, _ = O.isa_attention(Q, K, V, seg, 4, 0.4, 0.3, 0.2, gamma=-2.5)
    np.testing.assert_allclose(o2 - o0, -2.5 * (o1 - o0), rtol=0, atol=1e-13)
    # the selection does not depend on gamma
    _, p2 = O.isa_attention(Q, K, V, seg, 4, 0.4, 0.3, 0.2, gamma=-2.5)
    assert list(p1["kv_list"]) == list(p2["kv_list"]) and list(p1["full_list"]) == list(p2["full_list"])


def test_coarse_output_rows_are_convex_combinations_of_mean_values():
    rng = np.random.default_rng(8)
    seg = [21, 10]
    Q, K, V = rand_case(rng, seg, 6, qscale=3.0)
    _, plan = O.isa_attention(Q, K, V, seg, 4, 0.5, 0.5, gamma=0.7)
    oc, Vc = plan["O_coarse"], plan["Vc"]
    assert (oc <= Vc.max(axis=0) + 1e-14).all() and (oc >= Vc.min(axis=0) - 1e-14).all()
    # constant values: every convex combination is that constant, so the output is (1 + gamma) times it
    out, _ = O.isa_attention(Q, K, np.full_like(V, 2.0), seg, 4, 0.5, 0.5, 0.3, gamma=0.7)
    np.testing.assert_allclose(out, 2.0 * 1.7, rtol=0, atol=1e-13)


def test_coarse_output_closed_forms():
    rng = np.random.default_rng(9)
    seg = [12, 9]
    Q, K, V = rand_case(rng, seg, 4)
    # zero queries: uniform coarse map -> every row of O_coarse is the plain average of the mean values
    _, plan = O.isa_attention(Q * 0, K, V, seg, 4, 0.5, 0.5, gamma=1.0)
    np.testing.assert_allclose(plan["O_coarse"], np.tile(plan["Vc"].mean(axis=0), (plan["T"], 1)), atol=1e-15)
    # one-hot coarse map: row i of O_coarse is the mean value of the block it looks at
    T, D = 6, 8
    Kc = np.eye(T, D) * 50.0
    target = [3, 0, 5, 1, 1, 4]
    Qc = np.stack([Kc[c] for c in target])
    Vc = rng.standard_normal((T, 3))
    S = O.coarse_map(O.coarse_logits(Qc, Kc))
    np.testing.assert_allclose(O.coarse_output(S, Vc), Vc[target], atol=1e-12)
    # a transposed operand or a column softmax would fail this: asymmetric map, distinct values
    S2 = np.array([[0.9, 0.1], [0.2, 0.8]])
    np.testing.assert_allclose(O.coarse_output(S2, np.array([[1.0], [3.0]])), [[1.2], [2.6]], atol=1e-15)


# ------------------------------------------------------------------------------------------------
# the paper's other printed forms (READINGS): each switch does what its name says, on cases small enough to do by hand
# ------------------------------------------------------------------------------------------------
def _hand_case():
    """Two source blocks and three context blocks of one token each (block size 1), D = 4: pooled tensors = the tokens."""
    Q = np.array([[2.0, 0, 0, 0], [0, 2.0, 0, 0], [1, 1, 0, 0], [0, 0, 3.0, 0], [0, 0, 0, 1.0]])
    K = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [4.0, 0, 0, 0], [0, 1.0, 0, 0], [-1.0, -1.0, 0, 0]])
    V = np.arange(20, dtype=np.float64).reshape(5, 4)
    return Q, K, V, [2, 3]


def test_reading_of_the_pooled_map():
    Q, K, V, seg = _hand_case()
    raw = O.isa_plan(Q, K, V, seg, 1, 1 / 3, 0.4, readings={"coarse_map": "raw"})
    # raw reading: Eq. 1 on Q^c K^c^T itself: context columns of the source rows are [[8, 0, -2], [0, 2, -2]] -> means [4, 1, -2]
    np.testing.assert_allclose(raw["s_ctx"], [4.0, 1.0, -2.0], atol=1e-14)
    assert raw["kv_list"].tolist() == [0, 1, 2]
    # variance over the two source columns of Q K^T rows [2,0], [0,2], [1,1], [0,0], [0,0] = [1, 1, 0, 0, 0]
    np.testing.assert_allclose(raw["sharp"], [1.0, 1.0, 0.0, 0.0, 0.0], atol=1e-14)
    uns = O.isa_plan(Q, K, V, seg, 1, 1 / 3, 0.4, readings={"coarse_map": "softmax_unscaled"})
    row0 = np.exp([2.0, 0, 8.0, 0, -2.0]); row0 /= row0.sum()
    np.testing.assert_allclose(uns["S_coarse"][0], row0, rtol=1e-13)
    dflt = O.isa_plan(Q, K, V, seg, 1, 1 / 3, 0.4)
    row0 = np.exp(np.array([2.0, 0, 8.0, 0, -2.0]) / 2.0); row0 /= row0.sum()          # sqrt(D) = 2
    np.testing.assert_allclose(dflt["S_coarse"][0], row0, rtol=1e-13)
    # the pooled output of Stage 1 is an attention output under every reading
    np.testing.assert_allclose(raw["O_coarse"], dflt["O_coarse"], rtol=1e-13)
    with pytest.raises(ValueError):
        O.isa_plan(Q, K, V, seg, 1, 0.5, 0.5, readings={"coarse_map": "nonsense"})


def test_reading_of_the_kept_block_count():
    # context of 300 tokens in blocks of 128: 3 context blocks (one short) but only 2 whole ones
    assert O.keep_count_reading(0.5, [256, 300], 128, "floor_of_ratio_times_blocks") == 1          # floor(0.5 * 3)
    assert O.keep_count_reading(0.5, [256, 300], 128, "ratio_times_whole_blocks") == 1             # int(0.5 * 2)
    assert O.keep_count_reading(0.7, [256, 300], 128, "floor_of_ratio_times_blocks") == 2          # floor(2.1)
    assert O.keep_count_reading(0.7, [256, 300], 128, "ratio_times_whole_blocks") == 1             # int(1.4)
    # two references: the printed form pools the context length before dividing, the taken one cuts every reference
    assert O.keep_count_reading(1.0, [128, 100, 100], 128, "floor_of_ratio_times_blocks") == 2
    assert O.keep_count_reading(1.0, [128, 100, 100], 128, "ratio_times_whole_blocks") == 1
    rng = np.random.default_rng(3)
    Q, K, V = (rng.standard_normal((556, 8)) for _ in range(3))
    a = O.isa_plan(Q, K, V, [256, 300], 128, 0.7, 0.5)
    b = O.isa_plan(Q, K, V, [256, 300], 128, 0.7, 0.5, readings={"keep_rounding": "ratio_times_whole_blocks"})
    assert (a["k_keep"], b["k_keep"]) == (2, 1) and set(b["kv_list"]) <= set(a["kv_list"])


def test_reading_of_the_sharpness_columns():
    Q, K, V, seg = _hand_case()
    src = O.isa_plan(Q, K, V, seg, 1, 1.0, 0.4, readings={"coarse_map": "raw"})
    allc = O.isa_plan(Q, K, V, seg, 1, 1.0, 0.4, readings={"coarse_map": "raw", "sharpness_columns": "all"})
    rows = Q @ K.T
    np.testing.assert_allclose(allc["sharp"], rows.var(axis=1), rtol=1e-13)
    np.testing.assert_allclose(src["sharp"], rows[:, :2].var(axis=1), rtol=1e-13)
    # row 0 = [2, 0, 8, 0, -2]: flat over the source columns compared with row 1 = [0, 2, 0, 2, -2] only once the
    # context columns count
    assert allc["sharp"][0] > allc["sharp"][1] and src["sharp"][0] == src["sharp"][1]
