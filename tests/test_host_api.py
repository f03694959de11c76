"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, validates its
arguments and derives the same counts as the oracle.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import paper_2605_04569_amd as I
from oracle import isa_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "isa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(isa_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = I.lib()
    names = declared_symbols()
    assert "isa_attention" in names and "isa_dense_attention" in names and len(names) >= 12
    for n in names:
        assert hasattr(L, n), n


def base_problem(**kw):
    d = dict(H=2, D=64, dtype="f32", block=64, seg_len=[[512, 512]], keep_ratio=0.5, full_frac=0.25)
    d.update(kw)
    return I.Problem(**d)


def status(pr, **kw):
    cp, keep = pr.c_struct(**kw)
    out = I.binding._CCounts()
    return I.lib().isa_get_counts(C.byref(cp), 0, C.byref(out))


def test_validation_errors():
    assert status(base_problem()) == 0
    assert status(base_problem(D=96)) == -2
    assert status(base_problem(block=32)) == -2
    assert status(base_problem(seg_len=[[0, 512]])) == -2                  # empty source segment
    assert status(base_problem(seg_len=[[64] * 40])) == -2                 # too many segments
    assert status(base_problem(seg_len=[[64]] * 9)) == -2                  # too many batch items
    assert status(base_problem(keep_ratio=1.5)) == -3
    assert status(base_problem(full_frac=-0.1)) == -3
    assert status(base_problem(exact_frac=float("nan"))) == -3
    assert status(base_problem(dtype="f16")) == -4
    assert status(base_problem(gamma=0.1)) == 0
    assert status(base_problem(gamma=float("inf"))) == -5 and status(base_problem(gamma=float("nan"))) == -5
    assert status(base_problem(), strides=(0, 0, 60)) == -2                # stride_t < D
    assert status(base_problem(), strides=(8 * 1024 * 64, 1024 * 64 + 4, 64)) == -2
    assert I.lib().isa_get_counts(None, 0, None) == -1
    assert I.isa_workspace_bytes(base_problem(D=96)) == 0
    assert "RATIO" in I.isa_strerror(-3) and I.isa_strerror(0) == "ISA_OK" and "unknown" in I.isa_strerror(-99)


def test_null_and_workspace_errors_need_no_gpu():
    pr = base_problem()
    cp, keep = pr.c_struct()
    L = I.lib()
    one = C.c_void_p(256)   # non-null, 256-aligned dummy; never dereferenced because validation fails first
    assert L.isa_attention(C.byref(cp), None, one, one, one, one, 1 << 40, None) == -1
    assert L.isa_attention(C.byref(cp), one, one, one, one, None, 1 << 40, None) == -6
    assert L.isa_attention(C.byref(cp), one, one, one, one, C.c_void_p(264), 1 << 40, None) == -6
    assert L.isa_attention(C.byref(cp), one, one, one, one, one, 16, None) == -6
    assert L.isa_dense_attention(C.byref(cp), one, one, one, None, one, 1 << 40, None) == -1
    odd = C.c_void_p(264)   # 8-byte aligned only: token tensors are read 16 bytes at a time
    assert L.isa_attention(C.byref(cp), one, odd, one, one, one, 1 << 40, None) == -2
    assert L.isa_dense_attention(C.byref(cp), one, one, one, odd, one, 1 << 40, None) == -2
    assert L.isa_block_means(C.byref(cp), odd, one, one, one, one, one, one, 1 << 40, None) == -2
    assert L.isa_attention_simple(one, one, one, 2, 64, 0, 10, 0.5, 0.5, 64, one, None) == -2
    # the staged attend needs the coarse output exactly when gamma != 0
    cg, keep_g = base_problem(gamma=0.5).c_struct()
    assert L.isa_attend(C.byref(cg), one, one, one, one, one, one, one, one, None, None, one, one, 1 << 40, None) == -1
    assert L.isa_coarse_output(C.byref(cp), one, one, None, one, one, 1 << 40, None) == -1
    # a problem with a residual asks for room for the coarse output
    assert I.isa_workspace_bytes(base_problem(gamma=0.5)) > I.isa_workspace_bytes(base_problem())
    # backward pass: every tensor is required; the lists come all together or not at all; with exact sets the bits come
    # with them; shapes without MFMA kernels are unsupported (checked before the workspace is looked at)
    bw = L.isa_attention_backward
    mf, keep_m = base_problem(D=128, block=128, dtype="bf16").c_struct()
    assert bw(C.byref(mf), one, one, one, one, None, None, None, None, None, one, one, one, one, 1 << 40, None) == -1
    assert bw(C.byref(mf), one, one, one, one, one, None, None, None, None, one, one, None, one, 1 << 40, None) == -1
    assert bw(C.byref(mf), one, one, one, one, one, one, None, one, None, one, one, one, one, 1 << 40, None) == -1
    mx, keep_x = base_problem(D=128, block=128, dtype="bf16", exact_frac=0.25).c_struct()
    assert bw(C.byref(mx), one, one, one, one, one, one, one, one, None, one, one, one, one, 1 << 40, None) == -1
    assert bw(C.byref(cp), one, one, one, one, one, None, None, None, None, one, one, one, one, 1 << 40, None) == -5
    assert bw(C.byref(mf), one, one, one, one, one, None, None, None, None, one, one, one, None, 1 << 40, None) == -6
    assert bw(C.byref(mf), one, one, one, one, one, None, None, None, None, one, one, one, one, 16, None) == -6


def test_token_span_of_4_gib_is_refused_not_rerouted():
    """bf16, D = 128, block = 128 with the tokens of one head spanning 4 GiB or more (here q, k, v as views of a fused
    [S, 3, H, D] tensor at 720p): the matrix-core kernels cannot address it, and the call says so instead of running the
    portable kernels behind the caller's back; with those selected explicitly the problem is accepted."""
    pr = base_problem(H=40, D=128, block=128, dtype="bf16", seg_len=[[75600, 75600]])
    fused = (151200 * 3 * 40 * 128, 128, 3 * 40 * 128)
    assert status(pr) == 0 and status(pr, strides=fused) == -5
    cp, keep = pr.c_struct(strides=fused)
    assert I.lib().isa_workspace_bytes(C.byref(cp)) == 0
    prev = I.isa_set_mfma(False)
    try:
        assert status(pr, strides=fused) == 0
    finally:
        I.isa_set_mfma(prev)
    assert status(base_problem(H=40, D=128, block=128, dtype="bf16", seg_len=[[32760, 32760]]), strides=(65520 * 15360, 128, 15360)) == 0


def test_workspace_layout_is_consistent():
    """isa_workspace_layout: every array lies inside the workspace, 256-byte aligned, no two overlap; optional arrays
    are reported absent exactly when the problem does not have them."""
    for kw in (dict(), dict(exact_frac=0.25), dict(gamma=0.5), dict(D=128, block=128, dtype="bf16", exact_frac=0.1, gamma=1.0),
               dict(D=128, block=128, dtype="bf16", seg_len=[[700, 300, 41], [700, 900]])):
        pr = base_problem(**kw)
        lay = I.isa_workspace_layout(pr)
        assert lay["bytes"] == I.isa_workspace_bytes(pr)
        c = I.isa_get_counts(pr, 0)
        B, H, T, D = pr.B, pr.H, c["T_max"], pr.D
        size = dict(qc=B * H * T * D * 4, kc=B * H * T * D * 4, vc=B * H * T * D * 4, s_ctx=B * H * T * 4, sharp=B * H * T * 4,
                    kv_list=B * H * T * 4, full_list=B * H * T * 4, flat_list=B * H * T * 4,
                    exact_mask=B * H * T * ((T + 31) // 32) * 4, o_coarse=B * H * T * D * 4, nlse=B * H * pr.S_max * 4)
        assert (lay["exact_mask"] is None) == (pr.exact_frac == 0)
        assert (lay["o_coarse"] is None) == (pr.gamma == 0)
        assert (lay["nlse"] is None) == (not (pr.dtype == "bf16" and pr.D == 128 and pr.block == 128))
        spans = sorted((lay[n], lay[n] + size[n]) for n in size if lay[n] is not None)
        for lo, hi in spans:
            assert lo % 256 == 0 and hi <= lay["bytes"]
        for (lo0, hi0), (lo1, hi1) in zip(spans, spans[1:]):
            assert hi0 <= lo1
    bad, keep_b = base_problem(D=96).c_struct()
    assert I.lib().isa_workspace_layout(C.byref(bad), C.byref(I.binding._CLayout())) == -2
    ok, keep_o = base_problem().c_struct()
    assert I.lib().isa_workspace_layout(C.byref(ok), None) == -1


def test_static_scratch_entry_point_checks_before_it_touches_the_gpu():
    """isa_attention_static: argument errors and a problem whose forward-only workspace exceeds the library's fixed
    scratch array are refused before any HIP call."""
    L = I.lib()
    one = C.c_void_p(256)
    big, keep_b = base_problem(H=40, D=128, block=128, dtype="bf16", seg_len=[[32760, 32760]]).c_struct()
    assert L.isa_attention_static(C.byref(big), one, one, one, one, None) == -6
    assert L.isa_attention_static(C.byref(big), one, None, one, one, None) == -1
    assert L.isa_attention_static(C.byref(big), one, one, C.c_void_p(264), one, None) == -2
    bad, keep_x = base_problem(keep_ratio=2.0).c_struct()
    assert L.isa_attention_static(C.byref(bad), one, one, one, one, None) == -3


def test_prologue_validation_needs_no_gpu():
    L = I.lib()
    pr = base_problem()                                   # segments 512 + 512
    cp, keep = pr.c_struct()
    a = [C.c_void_p(256 * (i + 1)) for i in range(9)]     # never dereferenced: every case fails before a launch

    def call(grid, ptrs=None, means=(None, None, None)):
        cg, keep_g = grid.c_struct()
        ptrs = ptrs or a[:6]
        return L.isa_prologue(C.byref(cp), C.byref(cg), *ptrs, *means, None)

    good = dict(seg_grids=[[(4, 8, 16), (4, 8, 16)]], tile=(2, 4, 8), rope_dims=(16, 24, 24), rope_theta=10000.0)
    assert call(I.Grid(**{**good, "seg_grids": [[(4, 8, 16), (4, 8, 15)]]})) == -2          # grid != segment length
    assert call(I.Grid(**{**good, "tile": (2, 0, 8)})) == -2
    assert call(I.Grid(**{**good, "rope_dims": (16, 25, 23)})) == -2                        # odd
    assert call(I.Grid(**{**good, "rope_dims": (32, 24, 24)})) == -2                        # more than D = 64
    assert call(I.Grid(**{**good, "rope_dims": (-2, 24, 24)})) == -2
    assert call(I.Grid(**{**good, "rope_theta": 0.0})) == -5
    assert call(I.Grid(**{**good, "rope_theta": float("nan")})) == -5
    assert call(I.Grid(**good), ptrs=[a[0], a[1], a[2], a[3], a[4], None]) == -1
    assert call(I.Grid(**good), ptrs=[a[0], a[1], a[2], a[0], a[4], a[5]]) == -2            # output aliases an input
    assert call(I.Grid(**good), ptrs=[a[0], a[1], a[2], a[3], a[3], a[5]]) == -2            # two outputs alias
    assert call(I.Grid(**good), ptrs=[C.c_void_p(264), a[1], a[2], a[3], a[4], a[5]]) == -2  # not 16-byte aligned
    assert call(I.Grid(**good), means=(a[6], None, a[8])) == -1                             # means: all or none
    assert L.isa_prologue(C.byref(cp), None, *a[:6], None, None, None, None) == -1
    cg, keep_g = I.Grid(**good).c_struct()
    assert L.isa_prologue_backward(C.byref(cp), C.byref(cg), a[0], a[1], a[2], a[3], a[4], None, None) == -1
    assert L.isa_prologue_backward(C.byref(cp), C.byref(cg), a[0], a[1], a[2], a[1], a[4], a[5], None) == -2
    assert L.isa_untile(C.byref(cp), C.byref(cg), a[0], None, None) == -1
    assert L.isa_untile(C.byref(cp), C.byref(cg), a[0], a[0], None) == -2
    bad, keep_b = I.Grid(**{**good, "tile": (0, 1, 1)}).c_struct()
    assert L.isa_untile(C.byref(cp), C.byref(bad), a[0], a[1], None) == -2
    no_rope, keep_n = I.Grid(**{**good, "rope_theta": -1.0, "rope_dims": (1, 1, 1)}).c_struct()
    assert L.isa_untile(C.byref(cp), C.byref(no_rope), a[0], None, None) == -1             # embedding fields are not looked at


@pytest.mark.parametrize("seg,block,keep,full,exact", [
    ([[512, 512]], 64, 0.5, 0.25, 0.0),
    ([[7800, 7800]], 128, 0.5, 0.25, 0.0625),
    ([[32760, 1560, 32760], [32760, 17160]], 128, 0.75, 0.4, 0.0625),
    ([[75600, 75600]], 128, 0.5, 0.2, 0.0),
    ([[130]], 128, 0.3, 0.9, 0.5),
    ([[1000, 77, 1, 129]], 64, 0.1, 0.1, 0.1),
])
def test_counts_agree_with_oracle(seg, block, keep, full, exact):
    pr = base_problem(seg_len=seg, block=block, keep_ratio=keep, full_frac=full, exact_frac=exact)
    for b, s in enumerate(seg):
        c = I.isa_get_counts(pr, b)
        starts, counts, T_src = O.block_layout(s, block)
        T = len(starts)
        assert (c["S"], c["T"], c["T_src"], c["T_ctx"]) == (sum(s), T, T_src, T - T_src)
        assert c["k_keep"] == O.keep_count(keep, T - T_src) and c["T_new"] == T_src + c["k_keep"]
        assert (c["n_full"], c["n_flat"]) == O.group_counts(full, T)
        assert c["k_exact"] == O.exact_count(exact, c["T_new"])
    assert I.isa_workspace_bytes(pr) > 0
