"""The FLOP model bench.py reports against (algorithmic work of one step) checked against the paper's per-layer
formulas (App. B.2 / C.3, as coded in oracle/accounting.py) on the workloads where the paper's assumption a*d = h holds."""
import importlib.util
import os

import pytest

import synth
from oracle import accounting

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_step_flops_follow_the_papers_layer_formula(name):
    c = synth.CONFIGS[name]
    assert c["n_q_heads"] * c["head_dim"] == c["hidden"]
    s, b, h, m, a, k = c["seq"], c["batch"], c["hidden"], c["ffn"], c["n_q_heads"], c["n_kv_heads"]
    paper_fwd = accounting.fwd_flops(s, b, h, m, a, k)            # per layer, attention counted dense: 4 s^2 b h
    dense_attn = 4.0 * s * s * b * h
    proj = paper_fwd - dense_attn
    # bench: projections as the paper, causal attention = half of the dense count
    assert bench.fl_gemm_fwd(c) == pytest.approx(proj, rel=1e-12)
    layers, head = bench.algorithmic_flops(c)
    mult = 3.0 if c["train_base"] else 2.0                        # forward + two gradients (App. C.3), or one when frozen
    want = c["n_layers"] * (proj * mult + 0.5 * dense_attn * 3.5)  # attention backward = 2.5 x forward
    assert layers == pytest.approx(want, rel=1e-12)
    if c["vocab"]:
        assert head == pytest.approx(6.0 * s * b * h * c["vocab"], rel=1e-12)


def test_moe_flops_count_the_active_experts_only():
    c = synth.CONFIGS["C5"]
    T = c["batch"] * c["seq"]
    dense_like = dict(c, n_experts=0, top_k=0)
    extra = bench.fl_gemm_fwd(c) - bench.fl_gemm_fwd(dense_like)
    assert extra == pytest.approx(2.0 * T * (c["top_k"] - 1) * 3 * c["hidden"] * c["ffn"], rel=1e-12)
