"""Parity of isa_prologue / isa_untile (tile-order flattening, decoupled rotary embedding, fused block means) with the
fp64 oracle, element by element on small seeded cases and sampled at the 480p size.  All calls go through the C ABI."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import isa_oracle as O
from oracle import isa_oracle_prologue as P
from util import f64, problem_of

pytestmark = pytest.mark.gpu

CFG0 = W.CONFIGS["cfg0"]                                            # fp32, D = 64, block = 64, two 4x8x16 grids
SMALL_BF16 = W.CONFIGS["cfg1"].with_(name="small_bf16", H=5, src_grid=(2, 10, 33), ctx_grids=(((1, 10, 33), (1, 9, 20)),),
                                     seed=177)
RAGGED_B2 = W.CONFIGS["cfg3"].with_(name="ragged_b2", H=2, D=64, block=64, src_grid=(2, 9, 17),
                                    ctx_grids=(((1, 3, 5), (2, 9, 17)), ((1, 9, 17),)), seed=178)
SMALL_F32 = W.CONFIGS["cfg0"].with_(name="small_f32", H=3, D=128, block=128, src_grid=(3, 10, 23), ctx_grids=(((2, 10, 23),),),
                                    seed=179)
CASES = [CFG0, SMALL_BF16, RAGGED_B2, SMALL_F32]
ROPE = {64: (16, 24, 24), 128: (44, 42, 42)}     # the whole head turns; the axis borders fall inside a thread's chunk at D = 128
TILES = [(2, 4, 8), (2, 8, 8), (3, 5, 7), (1, 1, 4096)]


@pytest.fixture(scope="module")
def I():
    import paper_2605_04569_amd as isa
    isa.lib()                                     # fail loudly if the HIP library is not built
    return isa


def grids_of(wl):
    return [[wl.src_grid] + list(wl.ctx_grids[b]) for b in range(wl.B)]


def tolerances(wl, want):
    """Per-element bound: bf16 results are one rounding of an fp32 value that is itself within 1e-6 relative of the
    exact one, so they may land on the neighbouring bf16 number (2^-8 relative); fp32 results carry the error of the
    fp32 sine / cosine and of two products (a few 1e-7 of the pair's norm)."""
    if wl.dtype == "bf16":
        return 2.0 ** -8 * np.abs(want) + 1e-6 * np.abs(want).max()
    return 4e-6 * np.abs(want).max() * np.ones_like(want)


def run_prologue(I, wl, tile, rope_dims, theta=10000.0, means=True):
    Q, K, V = W.make_inputs(wl, "cpu")
    pr = problem_of(wl)
    grid = I.Grid(grids_of(wl), tile, rope_dims, theta)
    q, k, v = Q.cuda(), K.cuda(), V.cuda()
    qo, ko, vo = (torch.full_like(x, 7.0) for x in (q, k, v))
    T_max = I.isa_get_counts(pr, 0)["T_max"]
    mc = [torch.full((wl.B, wl.H, T_max, wl.D), -3.0, device="cuda") for _ in range(3)] if means else [None] * 3
    I.isa_prologue(pr, grid, q, k, v, qo, ko, vo, *mc)
    torch.cuda.synchronize()
    return pr, grid, (Q, K, V), (q, k, v), (qo, ko, vo), mc


@pytest.mark.parametrize("tile", TILES, ids=lambda t: "x".join(map(str, t)))
@pytest.mark.parametrize("wl", CASES, ids=lambda c: c.name)
def test_prologue_matches_oracle_everywhere(I, wl, tile):
    pr, grid, (Q, K, V), _, (qo, ko, vo), (qc, kc, vc) = run_prologue(I, wl, tile, ROPE[wl.D])
    rdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    for b in range(wl.B):
        n = wl.tokens(b)
        starts, counts, _ = O.block_layout(wl.seg_len(b), wl.block)
        for h in range(wl.H):
            want = P.prologue_head(f64(Q[b, h, :n]), f64(K[b, h, :n]), f64(V[b, h, :n]), grids_of(wl)[b], tile,
                                   ROPE[wl.D], 10000.0)
            for name, got_t, w, mean_t in (("q", qo, want[0], qc), ("k", ko, want[1], kc), ("v", vo, want[2], vc)):
                got = f64(got_t[b, h, :n])
                if name == "v":
                    assert np.array_equal(got, w), (wl.name, b, h)                     # a pure reordering: bit-exact
                else:
                    bad = np.abs(got - w) > tolerances(wl, w)
                    assert not bad.any(), (wl.name, name, b, h, int(bad.sum()), float(np.abs(got - w).max()))
                # the fused block means: means of the stored (rounded) values
                stored = f64(torch.from_numpy(w).to(rdt))
                wm = O.block_means(stored, starts, counts)
                gm = f64(mean_t[b, h, :len(starts)])
                atol = (2.0 ** -9 if wl.dtype == "bf16" else 4e-6) * np.abs(w).max()
                assert np.abs(gm - wm).max() <= atol, (wl.name, name, b, h, float(np.abs(gm - wm).max()))
            # rows past the batch item's tokens and means past its blocks are not written
            if n < qo.shape[2]:
                assert float((qo[b, h, n:] - 7.0).abs().max()) == 0.0
            if len(starts) < qc.shape[2]:
                assert float((qc[b, h, len(starts):] + 3.0).abs().max()) == 0.0


def test_partial_and_absent_embedding(I):
    wl = CFG0
    for dims in ((8, 0, 20), (0, 0, 0), (2, 2, 2)):
        _, _, (Q, K, V), _, (qo, ko, vo), _ = run_prologue(I, wl, (2, 4, 8), dims, theta=100.0, means=False)
        for h in range(wl.H):
            want = P.prologue_head(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), grids_of(wl)[0], (2, 4, 8), dims, 100.0)
            for got_t, w in ((qo, want[0]), (ko, want[1])):
                got = f64(got_t[0, h])
                assert not (np.abs(got - w) > tolerances(wl, w)).any()
                passed = sum(dims)                  # channels past the embedded ones are copied bit for bit
                assert np.array_equal(got[:, passed:], w[:, passed:])
            assert np.array_equal(f64(vo[0, h]), want[2])


@pytest.mark.parametrize("wl", [SMALL_BF16, RAGGED_B2, CFG0], ids=lambda c: c.name)
def test_untile_matches_oracle_and_inverts(I, wl):
    tile = (2, 4, 8)
    pr, grid, (Q, K, V), (q, k, v), (qo, ko, vo), _ = run_prologue(I, wl, tile, ROPE[wl.D], means=False)
    back = torch.full_like(vo, 9.0)
    I.isa_untile(pr, grid, vo, back)
    x = torch.full_like(v, 5.0)
    I.isa_untile(pr, grid, v, x)                  # any tensor: here the raster-order V read as if it were tile-ordered
    torch.cuda.synchronize()
    for b in range(wl.B):
        n = wl.tokens(b)
        for h in range(wl.H):
            assert torch.equal(back[b, h, :n], v[b, h, :n])                               # round trip
            want = P.untile_head(f64(V[b, h, :n]), grids_of(wl)[b], tile)
            assert np.array_equal(f64(x[b, h, :n]), want)
        if n < back.shape[2]:
            assert float((back[b, :, n:] - 9.0).abs().max()) == 0.0


@pytest.mark.parametrize("tile", [(2, 8, 8), (3, 5, 7)], ids=lambda t: "x".join(map(str, t)))
@pytest.mark.parametrize("wl", CASES, ids=lambda c: c.name)
def test_prologue_backward_matches_oracle_everywhere(I, wl, tile):
    """The transpose of the prologue on seeded gradients (the generator's Q, K, V stand in for dq_out, dk_out, dv_out)."""
    G = W.make_inputs(wl.with_(seed=wl.seed + 500), "cpu")
    pr = problem_of(wl)
    grid = I.Grid(grids_of(wl), tile, ROPE[wl.D], 10000.0)
    g_dev = [x.cuda() for x in G]
    d_in = [torch.full_like(x, 7.0) for x in g_dev]
    I.isa_prologue_backward(pr, grid, *g_dev, *d_in)
    torch.cuda.synchronize()
    for b in range(wl.B):
        n = wl.tokens(b)
        for h in range(wl.H):
            want = P.prologue_bwd_head(*(f64(x[b, h, :n]) for x in G), grids_of(wl)[b], tile, ROPE[wl.D], 10000.0)
            for name, got_t, w in zip("qkv", d_in, want):
                got = f64(got_t[b, h, :n])
                if name == "v":
                    assert np.array_equal(got, w), (wl.name, b, h)
                else:
                    bad = np.abs(got - w) > tolerances(wl, w)
                    assert not bad.any(), (wl.name, name, b, h, int(bad.sum()), float(np.abs(got - w).max()))
            if n < d_in[0].shape[2]:
                assert float((d_in[0][b, h, n:] - 7.0).abs().max()) == 0.0


def test_prologue_backward_inverts_the_prologue_at_full_size(I):
    """480p: the map is orthogonal, so the backward applied to the forward's output returns the input up to the two
    roundings to bf16 on the way (2^-8 relative of a pair's norm), and V bit for bit; sampled rows against the oracle."""
    wl = W.CONFIGS["cfg2"]
    tile, dims = (2, 8, 8), ROPE[128]
    pr = problem_of(wl)
    grid = I.Grid(grids_of(wl), tile, dims, 10000.0)
    q, k, v = W.make_inputs(wl, "cuda")
    qo, ko, vo = (torch.empty_like(x) for x in (q, k, v))
    I.isa_prologue(pr, grid, q, k, v, qo, ko, vo)
    qb, kb, vb = (torch.empty_like(x) for x in (q, k, v))
    I.isa_prologue_backward(pr, grid, qo, ko, vo, qb, kb, vb)
    torch.cuda.synchronize()
    assert torch.equal(vb, v)
    for x, xb in ((q, qb), (k, kb)):
        for h in (0, 21, 39):
            a, bb = x[0, h].float(), xb[0, h].float()
            norm = (a.view(-1, 64, 2) ** 2).sum(-1).sqrt().repeat_interleave(2, dim=1).view_as(a)
            assert bool(((a - bb).abs() <= 2.0 ** -7 * norm + 1e-6).all()), h
    g = wl.src_grid
    n_seg = g[0] * g[1] * g[2]
    perm = P.tile_order(g, tile)
    coords = P.grid_coords(g)
    rng = np.random.default_rng(6)
    rows = np.concatenate([[0, 1, 127, 128, n_seg - 1], rng.integers(0, n_seg, 200)])     # positions in tile order
    src = perm[rows]
    ang = P.rope_angles(coords[src], wl.D, dims, 10000.0)
    for h in (3, 38):
        for seg in range(2):
            want = P.rope_rotate(f64(qo[0, h, seg * n_seg + torch.from_numpy(rows).cuda()]), -ang)
            got = f64(qb[0, h, seg * n_seg + torch.from_numpy(src).cuda()])
            assert not (np.abs(got - want) > tolerances(wl, want)).any(), (h, seg)


def test_random_grids_and_tile_shapes(I):
    """The closed form that turns a position of the tile order into grid coordinates, against the oracle's explicit
    enumeration, over random grids and tile shapes (clipped tiles on any axis, tiles larger than the grid, one-token
    segments): V is a pure reordering, so every element must match bit for bit; Q is checked within the bound."""
    import random
    rng = random.Random(20260504)
    for case in range(60):
        n_seg = rng.randint(1, 3)
        grids = [(rng.randint(1, 5), rng.randint(1, 9), rng.randint(1, 21)) for _ in range(n_seg)]
        tile = (rng.randint(1, 4), rng.randint(1, 10), rng.randint(1, 12))
        wl = CFG0.with_(name="rand%d" % case, H=1, src_grid=grids[0], ctx_grids=(tuple(grids[1:]),), seed=300 + case)
        _, _, (Q, K, V), _, (qo, ko, vo), _ = run_prologue(I, wl, tile, ROPE[wl.D], means=False)
        want = P.prologue_head(f64(Q[0, 0]), f64(K[0, 0]), f64(V[0, 0]), grids, tile, ROPE[wl.D], 10000.0)
        assert np.array_equal(f64(vo[0, 0]), want[2]), (case, grids, tile)
        assert not (np.abs(f64(qo[0, 0]) - want[0]) > tolerances(wl, want[0])).any(), (case, grids, tile)


def test_fused_means_feed_the_staged_operator(I):
    """Prologue means -> isa_coarse_scores -> isa_select -> isa_attend gives what isa_attention computes from the
    prologue's outputs on its own (it recomputes the means in a different summation order)."""
    wl = SMALL_BF16.with_(keep_ratio=0.5, full_frac=0.3)
    pr, grid, _, _, (qo, ko, vo), (qc, kc, vc) = run_prologue(I, wl, (2, 8, 8), ROPE[wl.D])
    ws = I.new_workspace(pr)
    out_a = torch.zeros_like(qo)
    I.isa_attention(pr, qo, ko, vo, out_a, ws)
    T_max = qc.shape[2]
    f = dict(device="cuda", dtype=torch.float32)
    i = dict(device="cuda", dtype=torch.int32)
    s_ctx, sharp = torch.zeros((wl.B, wl.H, T_max), **f), torch.zeros((wl.B, wl.H, T_max), **f)
    kv, full, flat = (torch.full((wl.B, wl.H, T_max), -7, **i) for _ in range(3))
    qc2, kc2, vc2 = (torch.zeros_like(qc) for _ in range(3))
    ws2 = I.new_workspace(pr)
    I.isa_block_means(pr, qo, ko, vo, qc2, kc2, vc2, ws2)
    I.isa_coarse_scores(pr, qc, kc, s_ctx, sharp, None, ws2)
    I.isa_select(pr, s_ctx, sharp, None, kv, full, flat, None, ws2)
    out_b = torch.zeros_like(qo)
    I.isa_attend(pr, qo, ko, vo, kc, vc, kv, full, flat, None, out_b, ws2)
    torch.cuda.synchronize()
    for a, b2 in ((qc, qc2), (kc, kc2), (vc, vc2)):
        assert float((a - b2).abs().max()) <= 1e-5 * float(b2.abs().max())
    n = wl.tokens(0)
    d = (out_a[0, :, :n].float() - out_b[0, :, :n].float()).abs()
    assert float(d.max()) <= 2e-2 and float(d.mean()) <= 2e-3


def test_full_size_sampled(I):
    """480p (two 21x30x52 grids, 40 heads, bf16): sampled output rows against the oracle, the permutation property for
    V over the whole tensor, the fused means of sampled blocks."""
    wl = W.CONFIGS["cfg2"]
    tile, dims = (2, 8, 8), ROPE[128]
    pr = problem_of(wl)
    grid = I.Grid(grids_of(wl), tile, dims, 10000.0)
    q, k, v = W.make_inputs(wl, "cuda")
    qo, ko, vo = (torch.empty_like(x) for x in (q, k, v))
    T_max = I.isa_get_counts(pr, 0)["T_max"]
    qc, kc, vc = (torch.zeros((1, wl.H, T_max, wl.D), device="cuda") for _ in range(3))
    I.isa_prologue(pr, grid, q, k, v, qo, ko, vo, qc, kc, vc)
    torch.cuda.synchronize()
    g = wl.src_grid
    n_seg = g[0] * g[1] * g[2]
    perm = P.tile_order(g, tile)
    coords = P.grid_coords(g)
    perm_t = torch.from_numpy(perm).cuda()
    for seg in range(2):                           # V: the whole tensor, bit for bit
        assert torch.equal(vo[0, :, seg * n_seg:(seg + 1) * n_seg], v[0, :, seg * n_seg + perm_t])
    rng = np.random.default_rng(5)
    rows = np.concatenate([[0, 1, 127, 128, n_seg - 1], rng.integers(0, n_seg, 300)])
    starts, counts, _ = O.block_layout(wl.seg_len(0), wl.block)
    for h in (0, 17, 39):
        for seg in range(2):
            src = perm[rows]
            ang = P.rope_angles(coords[src], wl.D, dims, 10000.0)
            for x_in, x_out in ((q, qo), (k, ko)):
                want = P.rope_rotate(f64(x_in[0, h, seg * n_seg + torch.from_numpy(src).cuda()]), ang)
                got = f64(x_out[0, h, seg * n_seg + torch.from_numpy(rows).cuda()])
                assert not (np.abs(got - want) > tolerances(wl, want)).any(), (h, seg)
        for j in (0, 3, 255, 256, 300, len(starts) - 1):        # 255 / 511: the ragged last block of a segment
            seg, p0 = (0, starts[j]) if starts[j] < n_seg else (1, starts[j] - n_seg)
            src = perm[p0:p0 + counts[j]]
            ang = P.rope_angles(coords[src], wl.D, dims, 10000.0)
            idx = seg * n_seg + torch.from_numpy(src).cuda()
            for x_in, mean_t, rot in ((q, qc, True), (k, kc, True), (v, vc, False)):
                rows64 = f64(x_in[0, h, idx])
                w = P.rope_rotate(rows64, ang) if rot else rows64
                wm = f64(torch.from_numpy(w).to(torch.bfloat16)).mean(axis=0)
                assert np.abs(f64(mean_t[0, h, j]) - wm).max() <= 2.0 ** -9 * np.abs(w).max(), (h, j)


@pytest.mark.parametrize("wl", [SMALL_BF16, CFG0], ids=lambda c: c.name)
def test_prologue_then_operator_against_the_oracle_chain(I, wl):
    """Row-major, unrotated tensors -> isa_prologue -> isa_attention on the GPU, against the oracle's prologue (rounded to
    the storage type) followed by the oracle's operator: the lists the GPU chose must be valid selections of the oracle's
    scores and every output block must match the oracle evaluated on those lists."""
    from test_gpu_parity import check_end_to_end
    wl = wl.with_(keep_ratio=0.5, full_frac=0.3)
    tile = (2, 8, 8)
    pr, grid, (Q, K, V), _, (qo, ko, vo), _ = run_prologue(I, wl, tile, ROPE[wl.D], means=False)
    rdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    Qo, Ko, Vo = (torch.zeros_like(x) for x in (Q, K, V))
    for b in range(wl.B):
        n = wl.tokens(b)
        for h in range(wl.H):
            want = P.prologue_head(f64(Q[b, h, :n]), f64(K[b, h, :n]), f64(V[b, h, :n]), grids_of(wl)[b], tile,
                                   ROPE[wl.D], 10000.0)
            for dst, w in zip((Qo, Ko, Vo), want):
                dst[b, h, :n] = torch.from_numpy(w).to(rdt)
    # the two prologues may round an element to neighbouring bf16 values, so the means are not compared here
    a_kv, a_grp = check_end_to_end(I, wl, Qo, Ko, Vo, qo, ko, vo, check_means=False)
    assert a_kv >= 0.5 and a_grp >= 0.5


def test_maximum_block_count(I):
    """The library's limit of 4096 blocks (524 288 tokens in one segment, a 64x64x128 grid): V against the oracle's
    permutation over the whole tensor, sampled rows of Q, the last block's means, the round trip."""
    wl = W.CONFIGS["cfg1"].with_(name="max_blocks", H=2, src_grid=(64, 64, 128), ctx_grids=((),), seed=181)
    tile, dims = (4, 4, 8), ROPE[128]
    pr = problem_of(wl)
    assert I.isa_get_counts(pr, 0)["T"] == 4096
    grid = I.Grid(grids_of(wl), tile, dims, 10000.0)
    gen_ = torch.Generator(device="cuda").manual_seed(wl.seed)
    q, k, v = (torch.randn((1, wl.H, 524288, 128), generator=gen_, device="cuda").to(torch.bfloat16) for _ in range(3))
    qo, ko, vo = (torch.empty_like(x) for x in (q, k, v))
    qc, kc, vc = (torch.zeros((1, wl.H, 4096, 128), device="cuda") for _ in range(3))
    I.isa_prologue(pr, grid, q, k, v, qo, ko, vo, qc, kc, vc)
    back = torch.empty_like(v)
    I.isa_untile(pr, grid, vo, back)
    torch.cuda.synchronize()
    perm = P.tile_order(wl.src_grid, tile)
    assert torch.equal(vo[0], v[0][:, torch.from_numpy(perm).cuda()])
    assert torch.equal(back, v)
    coords = P.grid_coords(wl.src_grid)
    rows = np.concatenate([[0, 127, 128, 524287], np.random.default_rng(9).integers(0, 524288, 200)])
    src = perm[rows]
    ang = P.rope_angles(coords[src], 128, dims, 10000.0)
    for h in range(wl.H):
        want = P.rope_rotate(f64(q[0, h, torch.from_numpy(src).cuda()]), ang)
        got = f64(qo[0, h, torch.from_numpy(rows).cuda()])
        assert not (np.abs(got - want) > tolerances(wl, want)).any(), h
        src_last = perm[4095 * 128:]
        w = P.rope_rotate(f64(k[0, h, torch.from_numpy(src_last).cuda()]), P.rope_angles(coords[src_last], 128, dims, 10000.0))
        wm = f64(torch.from_numpy(w).to(torch.bfloat16)).mean(axis=0)
        assert np.abs(f64(kc[0, h, 4095]) - wm).max() <= 2.0 ** -9 * np.abs(w).max()


def test_prologue_operator_and_untile_replay_from_a_hip_graph(I):
    """The three calls only launch kernels on the caller's stream, so they can be captured together; every replay must
    reproduce the eager result bit for bit, also after the inputs change between replays."""
    wl = SMALL_BF16.with_(keep_ratio=0.5, full_frac=0.3)
    pr = problem_of(wl)
    grid = I.Grid(grids_of(wl), (2, 8, 8), ROPE[wl.D], 10000.0)
    Q, K, V = W.make_inputs(wl, "cpu")
    q, k, v = Q.cuda(), K.cuda(), V.cuda()
    ws = I.new_workspace(pr)

    def run(qi, ki, vi, bufs):
        qo, ko, vo, o_t, o_r = bufs
        I.isa_prologue(pr, grid, qi, ki, vi, qo, ko, vo)
        I.isa_attention(pr, qo, ko, vo, o_t, ws)
        I.isa_untile(pr, grid, o_t, o_r)

    eager = [torch.zeros_like(q) for _ in range(5)]
    run(q, k, v, eager)
    torch.cuda.synchronize()
    qs, ks, vs = q.clone(), k.clone(), v.clone()
    bufs = [torch.zeros_like(q) for _ in range(5)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(qs, ks, vs, bufs)                                        # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(qs, ks, vs, bufs)
    n = wl.tokens(0)
    for rep in range(3):
        bufs[4].zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(bufs[4][:, :, :n], eager[4][:, :, :n]), rep
        I.isa_dense_attention(pr, q, k, v, torch.empty_like(q), ws)   # eager work of our own between the replays
        torch.cuda.synchronize()
    qs.copy_(q.flip(1)); ks.copy_(k.flip(1)); vs.copy_(v.flip(1))
    graph.replay()
    torch.cuda.synchronize()
    eager2 = [torch.zeros_like(q) for _ in range(5)]
    run(q.flip(1).contiguous(), k.flip(1).contiguous(), v.flip(1).contiguous(), eager2)
    torch.cuda.synchronize()
    assert torch.equal(bufs[4][:, :, :n], eager2[4][:, :, :n])
