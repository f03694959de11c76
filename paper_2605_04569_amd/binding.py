"""ctypes binding of the C ABI in include/isa.h.

Argument marshalling only: every function here passes device pointers, sizes and the current
HIP stream to the entry point of the same name in libisa_hip.so.  There is no CPU fallback:
if the library has not been built, importing the binding's `lib()` raises.
"""
import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

ISA_BF16, ISA_F32 = 0, 1


def lib_path() -> str:
    return os.path.join(_HERE, "libisa_hip.so")


class IsaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (hip error %d)" % (where, isa_strerror(code), lib().isa_last_hip_error()))


class _CProblem(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("D", C.c_int32), ("dtype", C.c_int32), ("block", C.c_int32),
                ("seg_ptr", C.POINTER(C.c_int32)), ("seg_len", C.POINTER(C.c_int32)),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64),
                ("keep_ratio", C.c_double), ("full_frac", C.c_double), ("exact_frac", C.c_double), ("gamma", C.c_double)]


class _CGrid(C.Structure):
    _fields_ = [("seg_grid", C.POINTER(C.c_int32)), ("tile", C.c_int32 * 3), ("rope_dims", C.c_int32 * 3),
                ("rope_theta", C.c_double)]


class _CCounts(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("S", "T", "T_src", "T_ctx", "k_keep", "T_new", "n_flat", "n_full", "k_exact",
                                         "T_max")]


class _CLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("bytes", "qc", "kc", "vc", "s_ctx", "sharp", "kv_list", "full_list", "flat_list",
                                          "exact_mask", "o_coarse", "nlse")]


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2605_04569_amd.build)."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError("libisa_hip.so is not built: run __graft_entry__.build() "
                               "(there is no fallback path)")
        L = C.CDLL(path)
        P, V, ST, SZ = C.POINTER(_CProblem), C.c_void_p, C.c_void_p, C.c_size_t
        L.isa_get_counts.argtypes = [P, C.c_int, C.POINTER(_CCounts)]
        L.isa_workspace_bytes.argtypes = [P]
        L.isa_workspace_bytes.restype = C.c_size_t
        L.isa_workspace_layout.argtypes = [P, C.POINTER(_CLayout)]
        L.isa_attention.argtypes = [P, V, V, V, V, V, SZ, ST]
        L.isa_dense_attention.argtypes = [P, V, V, V, V, V, SZ, ST]
        L.isa_attention_static.argtypes = [P, V, V, V, V, ST]
        L.isa_attention_simple.argtypes = [V, V, V, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_double,
                                           C.c_int, V, ST]
        L.isa_block_means.argtypes = [P, V, V, V, V, V, V, V, SZ, ST]
        L.isa_coarse_scores.argtypes = [P, V, V, V, V, V, V, SZ, ST]
        L.isa_select.argtypes = [P, V, V, V, V, V, V, V, V, SZ, ST]
        L.isa_coarse_output.argtypes = [P, V, V, V, V, V, SZ, ST]
        L.isa_attend.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V, V, SZ, ST]
        L.isa_attention_backward.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V, V, V, SZ, ST]
        G = C.POINTER(_CGrid)
        L.isa_prologue.argtypes = [P, G, V, V, V, V, V, V, V, V, V, ST]
        L.isa_prologue_backward.argtypes = [P, G, V, V, V, V, V, V, ST]
        L.isa_untile.argtypes = [P, G, V, V, ST]
        L.isa_strerror.argtypes = [C.c_int]
        L.isa_strerror.restype = C.c_char_p
        L.isa_last_hip_error.argtypes = []
        L.isa_set_mfma.argtypes = [C.c_int]
        L.isa_time_attention_kernel.argtypes = [C.c_int]
        L.isa_last_attention_kernel_ms.argtypes = [C.POINTER(C.c_float)]
        _LIB = L
    return _LIB


@dataclass
class Problem:
    """Python mirror of isa_problem.  seg_len[b] lists batch item b's segments, source first."""
    H: int
    D: int
    dtype: str                       # "bf16" | "f32"
    block: int
    seg_len: Sequence[Sequence[int]]
    keep_ratio: float
    full_frac: float
    exact_frac: float = 0.0
    gamma: float = 0.0

    @property
    def B(self) -> int:
        return len(self.seg_len)

    @property
    def S_max(self) -> int:
        return max(sum(s) for s in self.seg_len)

    def c_struct(self, like: torch.Tensor = None, strides=None):
        """Returns (struct, keepalive).  Strides come from `like` ([B,H,S,D]) unless given."""
        flat: List[int] = []
        ptr = [0]
        for s in self.seg_len:
            flat += [int(x) for x in s]
            ptr.append(len(flat))
        a_ptr = (C.c_int32 * len(ptr))(*ptr)
        a_len = (C.c_int32 * max(1, len(flat)))(*flat)
        if strides is None:
            if like is not None:
                assert like.dim() == 4 and like.stride(3) == 1
                strides = (like.stride(0), like.stride(1), like.stride(2))
            else:
                strides = (self.H * self.S_max * self.D, self.S_max * self.D, self.D)
        cp = _CProblem(self.B, self.H, self.D, {"bf16": ISA_BF16, "f32": ISA_F32}.get(self.dtype, 99), self.block,
                       a_ptr, a_len, strides[0], strides[1], strides[2], self.keep_ratio, self.full_frac,
                       self.exact_frac, self.gamma)
        return cp, (a_ptr, a_len)


@dataclass
class Grid:
    """Python mirror of isa_grid.  seg_grids[b] lists the (t, h, w) grid of every segment of batch item b."""
    seg_grids: Sequence[Sequence[Sequence[int]]]
    tile: Sequence[int]
    rope_dims: Sequence[int] = (0, 0, 0)
    rope_theta: float = 10000.0

    def c_struct(self):
        flat: List[int] = []
        for grids in self.seg_grids:
            for g in grids:
                flat += [int(g[0]), int(g[1]), int(g[2])]
        arr = (C.c_int32 * max(1, len(flat)))(*flat)
        cg = _CGrid(arr, (C.c_int32 * 3)(*[int(x) for x in self.tile]),
                    (C.c_int32 * 3)(*[int(x) for x in self.rope_dims]), float(self.rope_theta))
        return cg, arr


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != 0:
        raise IsaError(rc, where)


def isa_strerror(code: int) -> str:
    return lib().isa_strerror(code).decode()


def isa_set_mfma(enabled: bool) -> int:
    return lib().isa_set_mfma(1 if enabled else 0)


def isa_time_attention_kernel(enabled: bool):
    _check(lib().isa_time_attention_kernel(1 if enabled else 0), "isa_time_attention_kernel")


def isa_last_attention_kernel_ms() -> float:
    ms = C.c_float()
    _check(lib().isa_last_attention_kernel_ms(C.byref(ms)), "isa_last_attention_kernel_ms")
    return ms.value


def isa_get_counts(pr: Problem, b: int = 0) -> dict:
    cp, keep = pr.c_struct()
    out = _CCounts()
    _check(lib().isa_get_counts(C.byref(cp), b, C.byref(out)), "isa_get_counts")
    return {n: getattr(out, n) for n, _ in _CCounts._fields_}


def isa_workspace_bytes(pr: Problem) -> int:
    cp, keep = pr.c_struct()
    return int(lib().isa_workspace_bytes(C.byref(cp)))


def isa_workspace_layout(pr: Problem) -> dict:
    """Byte offsets of the arrays isa_attention leaves in its workspace; None for arrays the problem does not have."""
    cp, keep = pr.c_struct()
    out = _CLayout()
    _check(lib().isa_workspace_layout(C.byref(cp), C.byref(out)), "isa_workspace_layout")
    none = C.c_size_t(-1).value
    return {n: (None if getattr(out, n) == none else int(getattr(out, n))) for n, _ in _CLayout._fields_}


def workspace_array(workspace: torch.Tensor, offset: int, shape, dtype: torch.dtype) -> torch.Tensor:
    """A view (no copy) of `shape` x `dtype` at byte `offset` of a workspace tensor."""
    n = 1
    for d in shape:
        n *= int(d)
    return workspace[offset:offset + n * torch.empty((), dtype=dtype).element_size()].view(dtype).view(*shape)


def new_workspace(pr: Problem, device="cuda") -> torch.Tensor:
    """A torch-owned device buffer of the size the library asks for (torch allocations are 256-byte aligned)."""
    return torch.empty(max(256, isa_workspace_bytes(pr)), dtype=torch.uint8, device=device)


def _same_layout(*ts):
    s = ts[0].stride()
    for t in ts:
        assert t.stride() == s and t.dtype == ts[0].dtype and t.is_cuda, "q, k, v, out must share dtype and strides"


def isa_attention(pr: Problem, q, k, v, out, workspace):
    _same_layout(q, k, v, out)
    cp, keep = pr.c_struct(q)
    _check(lib().isa_attention(C.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(workspace), workspace.numel(),
                               _stream()), "isa_attention")
    return out


def isa_attention_static(pr: Problem, q, k, v, out):
    _same_layout(q, k, v, out)
    cp, keep = pr.c_struct(q)
    _check(lib().isa_attention_static(C.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _stream()), "isa_attention_static")
    return out


def isa_dense_attention(pr: Problem, q, k, v, out, workspace):
    _same_layout(q, k, v, out)
    cp, keep = pr.c_struct(q)
    _check(lib().isa_dense_attention(C.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(workspace),
                                     workspace.numel(), _stream()), "isa_dense_attention")
    return out


def isa_attention_simple(q, k, v, n_src, n_ctx, keep_ratio, full_frac, block, out):
    H, S, D = q.shape
    assert S == n_src + n_ctx and q.is_contiguous() and k.is_contiguous() and v.is_contiguous() and out.is_contiguous()
    _check(lib().isa_attention_simple(_ptr(q), _ptr(k), _ptr(v), H, D, n_src, n_ctx, keep_ratio, full_frac, block,
                                      _ptr(out), _stream()), "isa_attention_simple")
    return out


def isa_block_means(pr: Problem, q, k, v, qc, kc, vc, workspace):
    _same_layout(q, k, v)
    cp, keep = pr.c_struct(q)
    _check(lib().isa_block_means(C.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(qc), _ptr(kc), _ptr(vc), _ptr(workspace),
                                 workspace.numel(), _stream()), "isa_block_means")


def isa_coarse_scores(pr: Problem, qc, kc, s_ctx, sharp, z, workspace):
    cp, keep = pr.c_struct()
    _check(lib().isa_coarse_scores(C.byref(cp), _ptr(qc), _ptr(kc), _ptr(s_ctx), _ptr(sharp), _ptr(z), _ptr(workspace),
                                   workspace.numel(), _stream()), "isa_coarse_scores")


def isa_coarse_output(pr: Problem, qc, kc, vc, o_coarse, workspace):
    cp, keep = pr.c_struct()
    _check(lib().isa_coarse_output(C.byref(cp), _ptr(qc), _ptr(kc), _ptr(vc), _ptr(o_coarse), _ptr(workspace),
                                   workspace.numel(), _stream()), "isa_coarse_output")


def isa_select(pr: Problem, s_ctx, sharp, z, kv_list, full_list, flat_list, exact_mask, workspace):
    cp, keep = pr.c_struct()
    _check(lib().isa_select(C.byref(cp), _ptr(s_ctx), _ptr(sharp), _ptr(z), _ptr(kv_list), _ptr(full_list),
                            _ptr(flat_list), _ptr(exact_mask), _ptr(workspace), workspace.numel(), _stream()),
           "isa_select")


def isa_attend(pr: Problem, q, k, v, kc, vc, kv_list, full_list, flat_list, exact_mask, out, workspace, o_coarse=None):
    _same_layout(q, k, v, out)
    cp, keep = pr.c_struct(q)
    _check(lib().isa_attend(C.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(kc), _ptr(vc), _ptr(kv_list), _ptr(full_list),
                            _ptr(flat_list), _ptr(exact_mask), _ptr(o_coarse), _ptr(out), _ptr(workspace), workspace.numel(),
                            _stream()), "isa_attend")
    return out


def isa_attention_backward(pr: Problem, q, k, v, out, d_out, dq, dk, dv, workspace, kv_list=None, full_list=None,
                           flat_list=None, exact_mask=None):
    _same_layout(q, k, v, out, d_out, dq, dk, dv)
    cp, keep = pr.c_struct(q)
    _check(lib().isa_attention_backward(C.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(d_out), _ptr(kv_list),
                                        _ptr(full_list), _ptr(flat_list), _ptr(exact_mask), _ptr(dq), _ptr(dk), _ptr(dv),
                                        _ptr(workspace),
                                        workspace.numel(), _stream()), "isa_attention_backward")
    return dq, dk, dv


def isa_prologue(pr: Problem, grid: Grid, q_in, k_in, v_in, q_out, k_out, v_out, qc=None, kc=None, vc=None):
    _same_layout(q_in, k_in, v_in, q_out, k_out, v_out)
    cp, keep = pr.c_struct(q_in)
    cg, keep_g = grid.c_struct()
    _check(lib().isa_prologue(C.byref(cp), C.byref(cg), _ptr(q_in), _ptr(k_in), _ptr(v_in), _ptr(q_out), _ptr(k_out),
                              _ptr(v_out), _ptr(qc), _ptr(kc), _ptr(vc), _stream()), "isa_prologue")
    return q_out, k_out, v_out


def isa_untile(pr: Problem, grid: Grid, x_tiled, x_raster):
    _same_layout(x_tiled, x_raster)
    cp, keep = pr.c_struct(x_tiled)
    cg, keep_g = grid.c_struct()
    _check(lib().isa_untile(C.byref(cp), C.byref(cg), _ptr(x_tiled), _ptr(x_raster), _stream()), "isa_untile")
    return x_raster


def isa_prologue_backward(pr: Problem, grid: Grid, dq_out, dk_out, dv_out, dq_in, dk_in, dv_in):
    _same_layout(dq_out, dk_out, dv_out, dq_in, dk_in, dv_in)
    cp, keep = pr.c_struct(dq_out)
    cg, keep_g = grid.c_struct()
    _check(lib().isa_prologue_backward(C.byref(cp), C.byref(cg), _ptr(dq_out), _ptr(dk_out), _ptr(dv_out), _ptr(dq_in),
                                       _ptr(dk_in), _ptr(dv_in), _stream()), "isa_prologue_backward")
    return dq_in, dk_in, dv_in
