"""The bf16-storage floor used by the full-size chain test (tests/storage_rounding.py), checked on the CPU: the wrapper
changes nothing but the rounding of stored tensors, undoes itself, and shows the effect the chain test relies on -- with
a residual stream fed by a small embedding, the q/k-path gradients of the last layer of a stage carry a visibly larger
error than the other weight gradients although no kernel is involved."""
import numpy as np

import parity_util as pu
import synth
from oracle import layers as L
from storage_rounding import bf16_storage


def test_wrapper_rounds_stored_tensors_and_restores_the_oracle():
    before = {n: getattr(L, n) for n in ("rmsnorm_fwd", "linear_fwd", "attention_bwd", "swiglu_bwd")}
    rng = np.random.default_rng(0)
    x = rng.standard_normal((16, 64)).astype(np.float32)
    W = rng.standard_normal((32, 64)).astype(np.float32)
    plain = L.linear_fwd(x, W)
    with bf16_storage():
        stored = L.linear_fwd(x, W)
        n, rstd = L.rmsnorm_fwd(x, np.ones(64, np.float32), 1e-6)
        heads, _ = L.rmsnorm_fwd(x.reshape(16, 2, 32), np.ones(32, np.float32), 1e-6)
    assert np.array_equal(stored, synth.bf16_round(plain))
    assert np.array_equal(n, synth.bf16_round(n)) and not np.array_equal(rstd, synth.bf16_round(rstd))
    assert not np.array_equal(heads, synth.bf16_round(heads))      # per-head norm: rounded after the rotation only
    assert all(getattr(L, k) is v for k, v in before.items())
    assert np.array_equal(L.linear_fwd(x, W), plain)


def test_storage_alone_puts_the_qk_path_gradients_above_the_others():
    c = dict(n_layers=3, hidden=512, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=1536, vocab=2048, n_experts=0, top_k=0,
             lora_rank=0, lora=(), train_base=1, batch=1, seq=256, x_from="emb")
    wl = synth.make_workload(c, 31)
    ref = pu.oracle_chain(c, wl, dtype=np.float32)
    with bf16_storage():
        flo = pu.oracle_chain(c, wl, dtype=np.float32)
    err = {n: pu.rel_l2(g, r) for n, g, r in pu.chain_pairs(ref, flo)}
    assert abs(flo["loss"] - ref["loss"]) / ref["loss"] < 1e-4
    assert 1e-3 < err["out"] < 2e-2 and all(v < 4e-2 for v in err.values())
    last = c["n_layers"] - 1
    for qk in ("Wq", "Wk"):
        assert err["L%d.%s" % (last, qk)] > 1.4 * err["L%d.Wo" % last], err
        assert err["L%d.%s" % (last, qk)] > 1.4 * err["L%d.Wv" % last], err
