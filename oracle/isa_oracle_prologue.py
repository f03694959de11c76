"""fp64 CPU oracle of the operator's prologue: tile-order flattening and decoupled rotary embedding.

TEST INFRASTRUCTURE ONLY.  Imported by the tests, by the smoke check and by the CPU-baseline leg of the benchmark, and
by nothing on the product path.  It shares no code with the HIP library and never calls it.

What it computes.  The tokens of every segment (the source video, each context reference) sit on a (t, h, w) grid and
arrive flattened row-major, w fastest.  The prologue
  1. rotates the channels of every query and key token by angles proportional to the token's grid coordinates, the
     coordinates counted from zero inside each segment (Sec. 4, "decoupled" rotary embedding: source and context are
     embedded independently, so neither the order nor the length of the other segments enters);
  2. reorders the tokens of every segment so that contiguous spatiotemporal tiles become contiguous runs of the
     sequence (Sec. 2 "Block Sparse Attention": tiles are formed first, then flattened in tile order, then the sequence
     is cut into blocks);
  3. optionally returns the block means of the result (Alg. 1 Stage 1), which is what the first stage of the operator
     would compute from it.
prologue_bwd_head is the transpose of steps 1-2 (the prologue's part of the backward pass)  [pinned: adjoint identity
against the forward, exact inverse because the map is orthogonal, one pair by hand].
Values are left untouched by step 1 (no positional rotation of V) and reordered by step 2.

Readings taken where the paper is silent (listed with their reasons in the design notes of this repository):

* tile shape (tt, th, tw) is a parameter; tiles are enumerated row-major over tile coordinates (w-tile fastest) and the
  tokens of a tile row-major over their coordinates inside it (w fastest); tiles at the far edges of a grid that the
  tile shape does not divide are clipped, i.e. simply hold fewer tokens  [pinned as a permutation: bijection, identity
  for degenerate tile shapes, every run of tt*th*tw tokens of a divisible grid is one box; the enumeration order itself
  is a reading];
* the rotary embedding is the usual one on interleaved channel pairs (2i, 2i+1), three-axis: the first d_t channels
  turn with the frame coordinate, the next d_h with the row, the next d_w with the column, channels beyond
  d_t + d_h + d_w pass through; pair j of an axis with d_a channels turns by  pos * theta^(-2j / d_a)  radians,
  counter-clockwise when the pair is read as (real, imaginary)  [pinned: identity at the origin of every segment,
  norm of every pair preserved, scores depend on coordinate differences only, hand value for one radian; channel
  split, base and pairing are a reading -- the paper names the embedding and the reset, not its layout].
"""
import numpy as np


def tile_order(grid, tile):
    """Raster indices of the tokens of a (t, h, w) grid, listed in tile order.

    Returns an int64 array `perm` of length t*h*w: position p of the tile-ordered sequence holds the token whose
    row-major (w fastest) index is perm[p].  Sec. 2 "Block Sparse Attention".
    """
    t, h, w = grid
    tt, th, tw = tile
    perm = []
    for t0 in range(0, t, tt):
        for h0 in range(0, h, th):
            for w0 in range(0, w, tw):
                for ft in range(t0, min(t0 + tt, t)):
                    for fh in range(h0, min(h0 + th, h)):
                        for fw in range(w0, min(w0 + tw, w)):
                            perm.append((ft * h + fh) * w + fw)
    return np.asarray(perm, dtype=np.int64)


def grid_coords(grid):
    """(t, h, w) coordinates of every token of a grid in row-major order, counted from zero: int64 [t*h*w, 3]."""
    t, h, w = grid
    out = np.empty((t * h * w, 3), dtype=np.int64)
    i = 0
    for ft in range(t):
        for fh in range(h):
            for fw in range(w):
                out[i] = (ft, fh, fw)
                i += 1
    return out


def rope_angles(coords, D, rope_dims, theta):
    """Rotation angle of every channel pair of every token: float64 [n, D/2]; zero for pairs that pass through.

    Sec. 4 (rotary embedding applied per segment with the coordinates reset to zero); layout as in the header.
    """
    coords = np.asarray(coords, dtype=np.float64)
    ang = np.zeros((coords.shape[0], D // 2), dtype=np.float64)
    pair = 0
    for axis in range(3):
        d_a = rope_dims[axis]
        for j in range(d_a // 2):
            ang[:, pair] = coords[:, axis] * float(theta) ** (-2.0 * j / d_a)
            pair += 1
    return ang


def rope_rotate(X, ang):
    """Rotate the interleaved channel pairs of X [n, D] by ang [n, D/2] radians, counter-clockwise."""
    X = np.asarray(X, dtype=np.float64)
    z = (X[:, 0::2] + 1j * X[:, 1::2]) * np.exp(1j * ang)
    out = np.empty_like(X)
    out[:, 0::2] = z.real
    out[:, 1::2] = z.imag
    return out


def prologue_head(Q, K, V, seg_grids, tile, rope_dims, theta):
    """The prologue for one (batch, head) slice.  Q, K, V [S, D] with the segments of seg_grids (a list of (t, h, w))
    one after the other, each row-major.  Returns (Q', K', V') [S, D] in tile order, Q' and K' rotated."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    D = Q.shape[1]
    outs = [np.empty_like(Q), np.empty_like(K), np.empty_like(V)]
    start = 0
    for grid in seg_grids:
        n = grid[0] * grid[1] * grid[2]
        ang = rope_angles(grid_coords(grid), D, rope_dims, theta)     # coordinates restart at zero in every segment
        perm = tile_order(grid, tile)
        outs[0][start:start + n] = rope_rotate(Q[start:start + n], ang)[perm]
        outs[1][start:start + n] = rope_rotate(K[start:start + n], ang)[perm]
        outs[2][start:start + n] = V[start:start + n][perm]
        start += n
    assert start == Q.shape[0]
    return tuple(outs)


def prologue_bwd_head(dQo, dKo, dVo, seg_grids, tile, rope_dims, theta):
    """Gradient of a loss with respect to the prologue's inputs, given its gradient with respect to the outputs, for one
    (batch, head) slice.  The prologue is linear: a rotation of every channel pair (Q, K only) followed by a reordering
    of the tokens, so its transpose puts row p back at its row-major place and turns every pair the other way.
    Returns (dQ, dK, dV) [S, D] in row-major order per segment."""
    dQo = np.asarray(dQo, dtype=np.float64)
    dKo = np.asarray(dKo, dtype=np.float64)
    dVo = np.asarray(dVo, dtype=np.float64)
    D = dQo.shape[1]
    outs = [np.empty_like(dQo), np.empty_like(dKo), np.empty_like(dVo)]
    start = 0
    for grid in seg_grids:
        n = grid[0] * grid[1] * grid[2]
        ang = rope_angles(grid_coords(grid), D, rope_dims, theta)
        perm = tile_order(grid, tile)
        for o, g, rotated in ((outs[0], dQo, True), (outs[1], dKo, True), (outs[2], dVo, False)):
            back = np.empty((n, D), dtype=np.float64)
            back[perm] = g[start:start + n]                    # row p of the tile order came from row perm[p]
            o[start:start + n] = rope_rotate(back, -ang) if rotated else back
        start += n
    assert start == dQo.shape[0]
    return tuple(outs)


def untile_head(X, seg_grids, tile):
    """Inverse reordering for one (batch, head) slice: X [S, D] in tile order -> row-major order per segment."""
    X = np.asarray(X)
    out = np.empty_like(X)
    start = 0
    for grid in seg_grids:
        n = grid[0] * grid[1] * grid[2]
        perm = tile_order(grid, tile)
        out[start + perm] = X[start:start + n]
        start += n
    return out
