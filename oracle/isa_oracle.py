"""fp64 CPU oracle of dense attention and of In-Context Sparse Attention (ISA).

TEST INFRASTRUCTURE ONLY.  This module is the yardstick the HIP kernels are
checked against.  It is imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark, and by nothing on the product path.  It
shares no code with the HIP library and never calls it.

Everything is plain numpy in float64, one (batch, head) slice at a time, with
no blocking, fusion or reordering beyond what the paper's definitions state.
Each function names the passage of the paper it follows.

Readings taken where the paper is silent or inconsistent (each is listed with
its reason in the design notes of this repository):

* blocks are aligned to segment starts (source, then every context reference);
  the last block of a segment may be short; block means run over real tokens
  only and a short block enters the Taylor sums with its real token count n_j
  in place of the nominal block length L_K   [pinned: the Taylor branch must
  be exact when all keys of a block coincide, short blocks included];
* the coarse map is a row softmax over all key blocks of Q^c K^c^T / sqrt(D)
  [parity unpinned: a reading of Sec. 2 "Pooling Attention" vs Alg. 1 Stage 1];
* the number of kept context blocks is floor(keep_ratio * T_ctx)
  [parity unpinned: Sec. 3 and Alg. 1 Stage 2 print different roundings];
* sharpness is the population variance over the source key columns of the
  all-column softmax row (Alg. 1 Stage 3) [parity unpinned: Sec. 3 "Grouped
  Computation" prints the variance over all columns];
* full_frac is the fraction of query blocks that receive exact attention; the
  count of Taylor blocks is floor((1 - full_frac) * T) as in Alg. 1 Stage 3
  with the algorithm's alpha_f read as 1 - full_frac;
* all rankings are by descending value with ties going to the lower index;
* the optional coarse residual gamma * O_coarse (Alg. 1 Stage 1 and Stage 5)
  adds block i's row of O_coarse = S_coarse V^c to every token of block i: the
  algorithm adds a [T, D] array to an [S, D] one without saying how
  [pinned as far as the mathematics goes: linear in gamma, rows of O_coarse
  are convex combinations of the mean values, closed forms for uniform and
  one-hot coarse maps; the broadcast itself is a reading].
"""
import math

import numpy as np


# --------------------------------------------------------------------------
# Standard attention (Sec. 2 "Standard Attention")
# --------------------------------------------------------------------------
def dense_attention(Q, K, V):
    """softmax(Q K^T / sqrt(D)) V for one head.  Q [N, D], K, V [S, D] -> [N, D]."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    logits = (Q @ K.T) / math.sqrt(Q.shape[1])
    logits = logits - logits.max(axis=1, keepdims=True)
    P = np.exp(logits)
    P = P / P.sum(axis=1, keepdims=True)
    return P @ V


# --------------------------------------------------------------------------
# Block partition (Sec. 2 "Block Sparse Attention"; Alg. 1 Stage 1)
# --------------------------------------------------------------------------
def block_layout(seg_len, block):
    """Cut every segment into blocks of `block` tokens from the segment start.

    seg_len: token counts, source segment first, then each context reference.
    Returns (starts, counts, T_src): token offset and real token count n_j of
    each block, and the number of source blocks.
    """
    seg_len = [int(x) for x in seg_len]
    block = int(block)
    if block < 1 or len(seg_len) < 1 or seg_len[0] < 1 or any(x < 0 for x in seg_len):
        raise ValueError("bad segments or block size")
    starts, counts = [], []
    offset = 0
    for length in seg_len:
        for s in range(0, length, block):
            starts.append(offset + s)
            counts.append(min(block, length - s))
        offset += length
    T_src = -(-seg_len[0] // block)
    return np.asarray(starts, dtype=np.int64), np.asarray(counts, dtype=np.int64), T_src


def block_means(X, starts, counts):
    """Q^c, K^c or V^c: arithmetic mean of each block's real tokens
    (Alg. 1 Stage 1; Alg. 2 Stage 1).  X [S, D] -> [T, D]."""
    X = np.asarray(X, dtype=np.float64)
    out = np.empty((len(starts), X.shape[1]), dtype=np.float64)
    for j, (s, n) in enumerate(zip(starts, counts)):
        out[j] = X[s:s + n].sum(axis=0) / float(n)
    return out


# --------------------------------------------------------------------------
# Pooling attention (Sec. 2 "Pooling Attention"; Alg. 1 Stage 1)
# --------------------------------------------------------------------------
def coarse_logits(Qc, Kc):
    """Z_ij = Q^c_i . K^c_j / sqrt(D)."""
    return (Qc @ Kc.T) / math.sqrt(Qc.shape[1])


def coarse_map(Z):
    """S_coarse: row softmax of the coarse logits over all T key blocks."""
    E = np.exp(Z - Z.max(axis=1, keepdims=True))
    return E / E.sum(axis=1, keepdims=True)


def coarse_output(S_coarse, Vc):
    """O_coarse = S_coarse V^c: the pooled attention output, one row per query
    block (Alg. 1 Stage 1).  -> [T, D]."""
    return np.asarray(S_coarse, dtype=np.float64) @ np.asarray(Vc, dtype=np.float64)


# --------------------------------------------------------------------------
# Pre-selection (Sec. 3 "Implementation of Pre-Selection", Eq. 1 and Eq. 2)
# --------------------------------------------------------------------------
def context_saliency(S_coarse, T_src):
    """Eq. 1: mean over the source query blocks of the coarse scores that
    fall on each context key block.  -> [T_ctx]."""
    return S_coarse[:T_src, T_src:].sum(axis=0) / float(T_src)


def keep_count(keep_ratio, T_ctx):
    """Number of context blocks kept by the Select Ratio."""
    return int(math.floor(float(keep_ratio) * T_ctx))


def top_indices(score, k):
    """Indices of the k largest entries, descending value, ties -> lower index."""
    score = np.asarray(score)
    order = sorted(range(len(score)), key=lambda j: (-score[j], j))
    return np.asarray(order[:k], dtype=np.int64)


def preselect(s_ctx, k_keep, T_src):
    """Eq. 2: key/value block list = every source block followed by the
    k_keep most salient context blocks, stored by ascending block index."""
    kept = np.sort(top_indices(s_ctx, k_keep))
    return np.concatenate([np.arange(T_src, dtype=np.int64), T_src + kept])


# --------------------------------------------------------------------------
# Query grouping (Sec. 3 "Grouped Computation"; Alg. 1 Stage 3)
# --------------------------------------------------------------------------
def sharpness(S_coarse, T_src):
    """M_i: population variance of row i of S_coarse over the source key
    columns, for every query block i (source and context alike)."""
    part = S_coarse[:, :T_src]
    mean = part.sum(axis=1, keepdims=True) / float(T_src)
    return ((part - mean) ** 2).sum(axis=1) / float(T_src)


def group_counts(full_frac, T):
    """(n_full, n_flat): how many query blocks get exact / Taylor attention."""
    n_flat = int(math.floor((1.0 - float(full_frac)) * T))
    return T - n_flat, n_flat


def group_queries(M, n_full):
    """Sort blocks by sharpness, descending; the first n_full go to the exact
    branch and the rest to the Taylor branch.  Both lists ascending."""
    order = top_indices(M, len(M))
    return np.sort(order[:n_full]), np.sort(order[n_full:])


# --------------------------------------------------------------------------
# Per-query-block exact set of the Taylor kernel (Alg. 2 Stage 2)
# --------------------------------------------------------------------------
def exact_count(exact_frac, T_new):
    return int(math.floor(float(exact_frac) * T_new))


def exact_set(Z_row, kv_list, k_exact):
    """The k_exact blocks of kv_list with the largest coarse logit for this
    query block; ties -> the block that comes earlier in kv_list."""
    pos = top_indices(np.asarray(Z_row)[kv_list], k_exact)
    return np.sort(np.asarray(kv_list)[pos])


# --------------------------------------------------------------------------
# The two attention branches (Alg. 1 Stage 4)
# --------------------------------------------------------------------------
def _tokens_of(blocks, starts, counts):
    if len(blocks) == 0:
        return np.zeros(0, dtype=np.int64)
    return np.concatenate([np.arange(starts[j], starts[j] + counts[j]) for j in blocks])


def full_branch(q, K, V, starts, counts, kv_list):
    """Exact softmax attention of the query rows q over every real token of
    every block in kv_list (K_new, V_new of Eq. 2)."""
    tok = _tokens_of(kv_list, starts, counts)
    return dense_attention(q, np.asarray(K, dtype=np.float64)[tok], np.asarray(V, dtype=np.float64)[tok])


def taylor_branch(q, K, V, Kc, Vc, starts, counts, kv_list, exact_blocks, return_parts=False):
    """Block-wise 0-th order Taylor attention for the query rows q
    (Sec. 3, Eq. 3 and Eq. 4; Alg. 2 Stage 3).

    Blocks of kv_list that are in exact_blocks contribute token by token
    (Eq. 3).  Every other block j of kv_list contributes one term built from
    its mean key and mean value, weighted by its token count n_j (Eq. 4).
    One max over all logits of a row is subtracted before exponentiation.
    With return_parts the un-normalised accumulator, the normaliser ell and the
    subtracted max are returned instead of their quotient.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    D = q.shape[1]
    scale = 1.0 / math.sqrt(D)
    exact_blocks = [int(j) for j in exact_blocks]
    mean_blocks = [int(j) for j in kv_list if int(j) not in set(exact_blocks)]
    tok = _tokens_of(exact_blocks, starts, counts)

    s_exact = (q @ K[tok].T) * scale                       # [nq, n_tok]
    s_mean = (q @ Kc[mean_blocks].T) * scale               # [nq, n_mean]
    m = np.full((q.shape[0], 1), -np.inf)
    if s_exact.shape[1]:
        m = np.maximum(m, s_exact.max(axis=1, keepdims=True))
    if s_mean.shape[1]:
        m = np.maximum(m, s_mean.max(axis=1, keepdims=True))
    p_exact = np.exp(s_exact - m)
    p_mean = np.exp(s_mean - m) * counts[mean_blocks].astype(np.float64)[None, :]
    ell = p_exact.sum(axis=1, keepdims=True) + p_mean.sum(axis=1, keepdims=True)
    acc = p_exact @ V[tok] + p_mean @ Vc[mean_blocks]
    if return_parts:
        return acc, ell, m
    return acc / ell


# --------------------------------------------------------------------------
# Whole operator for one (batch, head) slice (Alg. 1)
# --------------------------------------------------------------------------
# The places where the paper prints two different things, and the alternative to the reading this oracle (and the HIP
# path) takes.  The alternatives exist to measure what the choice changes (design notes); nothing else uses them.
READINGS = {
    # pooled map used by Eq. 1 and by the sharpness: "softmax_scaled" = row softmax of Q^c K^c^T / sqrt(D) (taken: Sec. 2
    # "Pooling Attention" says standard attention is performed on the pooled tensors); "softmax_unscaled" = the formula as
    # printed there, softmax(Q^c K^c^T) without the 1 / sqrt(D); "raw" = Alg. 1 Stage 1 as printed, Q^c K^c^T with neither
    "coarse_map": ("softmax_scaled", "softmax_unscaled", "raw"),
    # kept context blocks: "floor_of_ratio_times_blocks" = floor(alpha_s * T_ctx) with T_ctx the number of context blocks,
    # short tail blocks included (taken; Sec. 3 prints alpha_s * ceil(L_ctx / b)); "ratio_times_whole_blocks" = Alg. 1
    # Stage 2 as printed, alpha_s * int(L_ctx / b), the product cut to an integer
    "keep_rounding": ("floor_of_ratio_times_blocks", "ratio_times_whole_blocks"),
    # columns of a pooled row whose variance is the sharpness: "source" (taken; Alg. 1 Stage 3 slices the source key
    # blocks) or "all" (Sec. 3 "Grouped Computation" prints the variance of the whole row)
    "sharpness_columns": ("source", "all"),
}


def pooled_map(Z_scaled, D, reading):
    """The pooled attention map under one of the READINGS["coarse_map"]; Z_scaled = Q^c K^c^T / sqrt(D)."""
    if reading == "softmax_scaled":
        return coarse_map(Z_scaled)
    if reading == "softmax_unscaled":
        return coarse_map(Z_scaled * math.sqrt(D))
    if reading == "raw":
        return Z_scaled * math.sqrt(D)
    raise ValueError(reading)


def keep_count_reading(keep_ratio, seg_len, block, reading):
    """Kept context blocks under one of the READINGS["keep_rounding"]."""
    ctx = [int(x) for x in seg_len[1:]]
    if reading == "floor_of_ratio_times_blocks":
        return keep_count(keep_ratio, sum(-(-x // block) for x in ctx))
    if reading == "ratio_times_whole_blocks":
        return int(float(keep_ratio) * (sum(ctx) // block))
    raise ValueError(reading)


def isa_plan(Q, K, V, seg_len, block, keep_ratio, full_frac, exact_frac=0.0, gamma=0.0, readings=None):
    """Stages 1-3 of Alg. 1: everything up to and including the index lists,
    plus the coarse output O_coarse and the stacking factor gamma that Stage 5
    uses.  `readings` (a dict over the keys of READINGS) swaps in the paper's
    other printed form at the places where it prints two; the default is the
    reading documented in the header, the one the HIP path implements."""
    rd = {k: v[0] for k, v in READINGS.items()}
    rd.update(readings or {})
    for k, v in rd.items():
        if v not in READINGS[k]:
            raise ValueError("unknown reading %s=%s" % (k, v))
    starts, counts, T_src = block_layout(seg_len, block)
    T = len(starts)
    Qc = block_means(Q, starts, counts)
    Kc = block_means(K, starts, counts)
    Vc = block_means(V, starts, counts)
    Z = coarse_logits(Qc, Kc)
    S = pooled_map(Z, Qc.shape[1], rd["coarse_map"])
    s_ctx = context_saliency(S, T_src)
    k_keep = min(T - T_src, keep_count_reading(keep_ratio, seg_len, block, rd["keep_rounding"]))
    kv_list = preselect(s_ctx, k_keep, T_src)
    M = sharpness(S, T_src if rd["sharpness_columns"] == "source" else T)
    n_full, n_flat = group_counts(full_frac, T)
    full_list, flat_list = group_queries(M, n_full)
    S_softmax = S if rd["coarse_map"] == "softmax_scaled" else coarse_map(Z)       # Stage 1's O_coarse is attention output
    return dict(starts=starts, counts=counts, T_src=T_src, T=T, Qc=Qc, Kc=Kc, Vc=Vc, Z=Z,
                S_coarse=S, O_coarse=coarse_output(S_softmax, Vc), gamma=float(gamma), s_ctx=s_ctx, k_keep=k_keep, kv_list=kv_list, sharp=M,
                n_full=n_full, n_flat=n_flat, full_list=full_list, flat_list=flat_list,
                exact_frac=float(exact_frac), k_exact=exact_count(exact_frac, len(kv_list)), readings=rd)


def attend_block(i, plan, Q, K, V, kv_list=None, in_full=None, exact_blocks=None):
    """Stage 4 for the tokens of query block i, plus the coarse residual of
    Stage 5: gamma times block i's row of O_coarse is added to each of its
    tokens (O_coarse has one row per block, the output one per token; reading:
    a block's row is shared by its tokens).  The index lists default to the
    plan's own; a caller may substitute lists produced elsewhere."""
    starts, counts = plan["starts"], plan["counts"]
    kv_list = plan["kv_list"] if kv_list is None else np.asarray(kv_list, dtype=np.int64)
    if in_full is None:
        in_full = bool(np.any(plan["full_list"] == i))
    q = np.asarray(Q, dtype=np.float64)[starts[i]:starts[i] + counts[i]]
    res = plan["gamma"] * plan["O_coarse"][i][None, :] if plan["gamma"] != 0.0 else 0.0
    if in_full:
        return full_branch(q, K, V, starts, counts, kv_list) + res
    if exact_blocks is None:
        exact_blocks = exact_set(plan["Z"][i], kv_list, exact_count(plan["exact_frac"], len(kv_list)))
    return taylor_branch(q, K, V, plan["Kc"], plan["Vc"], starts, counts, kv_list, exact_blocks) + res


def isa_attention(Q, K, V, seg_len, block, keep_ratio, full_frac, exact_frac=0.0, gamma=0.0):
    """Alg. 1 for one (batch, head) slice.  Q, K, V [S, D].
    Returns (out [S, D], plan)."""
    plan = isa_plan(Q, K, V, seg_len, block, keep_ratio, full_frac, exact_frac, gamma)
    out = np.zeros((np.asarray(Q).shape[0], np.asarray(V).shape[1]), dtype=np.float64)
    for i in range(plan["T"]):
        s, n = plan["starts"][i], plan["counts"][i]
        out[s:s + n] = attend_block(i, plan, Q, K, V)          # Stage 5: rows land in token order
    return out, plan
