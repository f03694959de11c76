"""torch.autograd glue over the C ABI: isa_attention as a differentiable function of q, k, v.

Plumbing only: the forward is one isa_attention call, the backward one isa_attention_backward call on the workspace
the forward left its lists and log-sum-exps in.  Gradients follow the library's definition: the index decisions of
Alg. 1 Stages 2-3 are held fixed, everything else (block means of the Taylor branch, the coarse residual) is
differentiated.  Only the shapes the backward kernels cover: bf16, D = 128, block = 128.
"""
import torch

from . import binding as B


class _IsaAttentionFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, problem, workspace):
        out = torch.empty_like(q)
        if q.shape[0] > 1 or problem.S_max < q.shape[2]:
            out.zero_()                          # rows past a batch item's end are not written by the library
        B.isa_attention(problem, q, k, v, out, workspace)
        ctx.save_for_backward(q, k, v, out)
        ctx.problem, ctx.workspace = problem, workspace
        return out

    @staticmethod
    def backward(ctx, d_out):
        q, k, v, out = ctx.saved_tensors
        if d_out.stride() != q.stride():         # the library wants one layout for all seven tensors
            g = torch.empty_like(q)
            g.copy_(d_out)
            d_out = g
        dq, dk, dv = (torch.zeros_like(q) for _ in range(3))
        B.isa_attention_backward(ctx.problem, q, k, v, out, d_out, dq, dk, dv, ctx.workspace)
        return dq, dk, dv, None, None


class InContextSparseAttention(torch.nn.Module):
    """ISA (Alg. 1) over [B, H, S, D] tensors (any strides with a contiguous last dimension; q, k, v alike) whose tokens
    are the source segment followed by the context references of `seg_len`.

    The module owns one workspace, sized at the first call and whenever the problem grows; the backward pass reads what
    the forward pass left there, so a module instance serves one forward/backward pair at a time (one instance per layer
    in a model; not reentrant, and a second forward before the backward of the first invalidates the first's gradients).
    """

    def __init__(self, seg_len, keep_ratio=0.125, full_frac=0.5, exact_frac=0.0625, gamma=0.0, block=128):
        super().__init__()
        self.seg_len = [list(s) for s in seg_len]
        self.ratios = dict(keep_ratio=keep_ratio, full_frac=full_frac, exact_frac=exact_frac, gamma=gamma)
        self.block = block
        self._workspace = None

    def forward(self, q, k, v):
        assert q.dim() == 4 and q.dtype == torch.bfloat16 and q.shape[3] == 128 and self.block == 128, \
            "the differentiable path covers bf16, D = 128, block = 128"
        assert q.shape[0] == len(self.seg_len)
        pr = B.Problem(H=q.shape[1], D=q.shape[3], dtype="bf16", block=self.block, seg_len=self.seg_len, **self.ratios)
        need = B.isa_workspace_bytes(pr)
        if self._workspace is None or self._workspace.numel() < need or self._workspace.device != q.device:
            self._workspace = torch.empty(max(256, need), dtype=torch.uint8, device=q.device)
        if k.stride() != q.stride():
            k = k.contiguous() if q.is_contiguous() else torch.empty_like(q).copy_(k)
        if v.stride() != q.stride():
            v = v.contiguous() if q.is_contiguous() else torch.empty_like(q).copy_(v)
        return _IsaAttentionFunction.apply(q, k, v, pr, self._workspace)
