"""The synthetic-input recipe: shapes, determinism and the statistics it promises."""
import math

import torch

import workloads as W


def test_config_shapes():
    assert W.CONFIGS["cfg0"].seg_len(0) == [512, 512]
    assert W.CONFIGS["cfg1"].seg_len(0) == [7800, 7800]
    assert W.CONFIGS["cfg2"].seg_len(0) == [32760, 32760]
    assert W.CONFIGS["cfg3"].seg_len(0) == [32760, 1560, 32760]
    assert W.CONFIGS["cfg3"].seg_len(1) == [32760, 17160]
    assert W.CONFIGS["cfg4"].seg_len(0) == [75600, 75600]
    assert W.CONFIGS["cfg3"].S_max == 67080


def test_cfg0_is_deterministic_and_has_the_promised_statistics():
    wl = W.CONFIGS["cfg0"]
    Q, K, V = W.make_inputs(wl)
    Q2, K2, V2 = W.make_inputs(wl)
    assert torch.equal(Q, Q2) and torch.equal(K, K2) and torch.equal(V, V2)
    assert Q.shape == (1, 2, 1024, 64) and Q.dtype == torch.float32
    n_src = 512
    # smooth field (unit std) + 0.3 noise -> std sqrt(1.09); context keys halved
    # (per field, i.e. per head, channel and segment, around the field's own mean)
    def field_std(x):
        return x.std(dim=2, unbiased=False).mean().item()
    assert abs(field_std(V[:, :, :n_src]) - math.sqrt(1.09)) < 0.05
    assert abs(field_std(K[:, :, :n_src]) - math.sqrt(1.09)) < 0.05
    assert abs(field_std(K[:, :, n_src:]) - 0.5 * math.sqrt(1.09)) < 0.05
    # neighbouring tokens along w are strongly correlated (sigma = 2 tokens)
    v = V[0, 0, :n_src, 0].view(4, 8, 16)
    c = torch.corrcoef(torch.stack([v[:, :, :-1].flatten(), v[:, :, 1:].flatten()]))[0, 1].item()
    assert c > 0.6
    # query norms spread over the log-uniform factor range
    qn = Q.norm(dim=-1) / math.sqrt(64)
    assert 0.3 < qn.min().item() < 0.8 and 3.0 < qn.max().item() < 5.5


def test_ragged_batch_rows_past_the_end_are_zero():
    wl = W.CONFIGS["cfg3"].with_(H=1, D=8, src_grid=(1, 3, 5), ctx_grids=(((1, 2, 3), (2, 3, 5)), ((1, 3, 5),)))
    Q, K, V = W.make_inputs(wl)
    assert Q.shape == (2, 1, 51, 8) and Q.dtype == torch.bfloat16
    assert wl.tokens(1) == 30
    assert torch.count_nonzero(Q[1, :, 30:]) == 0 and torch.count_nonzero(K[1, :, 30:]) == 0
