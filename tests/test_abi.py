"""CPU-side checks of the C-ABI library: it loads, exports every symbol the headers declare, and its pure host
functions (sizes, layouts, argument validation) behave.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2604_27085_amd", "librp.so")
if not os.path.exists(LIB):
    import __graft_entry__
    __graft_entry__.build()

from paper_2604_27085_amd import binding as B  # noqa: E402
from paper_2604_27085_amd import harness as H  # noqa: E402


def declared_symbols():
    names = []
    for hdr in ("rp.h", "rp_ops.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        names += re.findall(r"RP_API\s+[\w\s\*]+?\b(rp_\w+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 21
    for n in names:
        assert hasattr(B.lib, n), n
    assert sorted(B.EXPORTS) == names


@pytest.mark.parametrize("name", sorted(synth.CONFIGS))
def test_layouts_are_packed_and_disjoint(name):
    c = synth.CONFIGS[name]
    cfg = H.cfg_from_dict(c)
    wbytes, gbytes, wsbytes = B.rp_query_sizes(cfg, c["batch"], c["seq"])
    assert wsbytes > 0 and wbytes % 256 == 0 and gbytes % 256 == 0
    for query, es, total in ((B.rp_weight_layout, 2, wbytes), (B.rp_grad_layout, 4, gbytes)):
        spans = []
        for layer in range(cfg.n_layers + 1):
            for tid in range(len(B.TENSOR_IDS)):
                off, n = query(cfg, layer, tid)
                if n:
                    assert off % 16 == 0
                    spans.append((off, off + n * es))
        spans.sort()
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0
        assert not spans or spans[-1][1] <= total
    # chunk ranges tile the blob
    end_prev = 0
    for layer in range(cfg.n_layers + 1):
        b, e = B.rp_weight_chunk(cfg, layer)
        assert b == end_prev and e >= b
        end_prev = e
    assert end_prev == wbytes
    # the paper's upload-volume formula (App. C.1, Eq. bytes-dense, per layer, without the activation term) holds
    # whenever a*d == h, up to the norm gains and adapters it leaves out
    if c["n_q_heads"] * c["head_dim"] == c["hidden"] and c["n_experts"] == 0:
        h, m, a, k = c["hidden"], c["ffn"], c["n_q_heads"], c["n_kv_heads"]
        paper = 4 * h * h + 4 * h * h * k / a + 6 * h * m
        b, e = B.rp_weight_chunk(cfg, 0)
        small = 2 * (2 * h + 2 * c["head_dim"]) + 2 * c["lora_rank"] * 2 * sum(
            {"q": 2 * h, "k": h + h * k // a, "v": h + h * k // a, "o": 2 * h, "gate": h + m, "up": h + m, "down": h + m}[n]
            for n in c["lora"]) + 256
        assert paper <= e - b <= paper + small


def test_frozen_base_gradient_blob_holds_only_adapters():
    c = synth.CONFIGS["C3"]
    cfg = H.cfg_from_dict(c)
    assert B.rp_grad_layout(cfg, 0, B.T["WQKV"])[1] == 0
    assert B.rp_grad_layout(cfg, 0, B.T["LA_DOWN"])[1] == 16 * c["ffn"]
    # adapted A matrices of a fused projection are adjacent (one product fills them)
    oq, nq = B.rp_grad_layout(cfg, 1, B.T["LA_Q"])
    ok, nk = B.rp_grad_layout(cfg, 1, B.T["LA_K"])
    ov, _ = B.rp_grad_layout(cfg, 1, B.T["LA_V"])
    assert ok == oq + 4 * nq and ov == ok + 4 * nk


def test_pack_roundtrip_places_values():
    c = synth.CONFIGS["C1"]
    cfg = H.cfg_from_dict(c)
    wl = synth.make_workload(c, 3)
    blob = H.pack_weights(cfg, wl["layers"], wl["head"]).view(np.uint16)
    off, n = B.rp_weight_layout(cfg, 1, B.T["WQKV"])
    got = synth.bits_to_f32(blob[off // 2: off // 2 + n]).reshape(512, 256)
    np.testing.assert_array_equal(got[:256], wl["layers"][1]["Wq"])
    np.testing.assert_array_equal(got[384:], wl["layers"][1]["Wv"])
    off, n = B.rp_weight_layout(cfg, 2, B.T["WV"])
    np.testing.assert_array_equal(synth.bits_to_f32(blob[off // 2: off // 2 + n]).reshape(4096, 256), wl["head"]["Wv"])
    off, n = B.rp_weight_layout(cfg, 0, B.T["LB_V"])
    np.testing.assert_array_equal(synth.bits_to_f32(blob[off // 2: off // 2 + n]).reshape(128, 8), wl["layers"][0]["lora"]["v"][1])


def test_argument_validation_returns_codes_without_gpu():
    c = dict(synth.CONFIGS["C1"])
    good = H.cfg_from_dict(c)
    bad = H.cfg_from_dict(c)
    bad.struct_size = 12
    with pytest.raises(B.RpError) as e:
        B.rp_query_sizes(bad, 1, 128)
    assert e.value.code == B.RP_EINVAL
    for key, val, code in (("head_dim", 96, B.RP_EUNSUPPORTED), ("hidden", 260, B.RP_EUNSUPPORTED),
                           ("n_kv_heads", 3, B.RP_EINVAL), ("lora_rank", 12, B.RP_EUNSUPPORTED)):
        cc = dict(c)
        cc[key] = val
        with pytest.raises(B.RpError) as e:
            B.rp_query_sizes(H.cfg_from_dict(cc), 1, 128)
        assert e.value.code == code, key
    with pytest.raises(B.RpError) as e:
        B.rp_query_sizes(good, 1, 100)          # T not a multiple of 8
    assert e.value.code == B.RP_EUNSUPPORTED
    with pytest.raises(B.RpError) as e:
        B.rp_weight_layout(good, 7, 0)
    assert e.value.code == B.RP_EINVAL
    # NULL ctx is rejected by every stage call before anything else happens
    assert B.lib.rp_stage_forward(None, 0, None, None, None, None, 1, 8, None, 0) == B.RP_EINVAL
    assert B.lib.rp_stage_backward(None, 0, 3, None, None, None, None, None, None, None, 1, 8, None, 0) == B.RP_EINVAL
    assert B.lib.rp_lmhead_ce_fwd_bwd(None, 0, None, None, None, None, None, 1.0, 1, 8, None, 0) == B.RP_EINVAL
    assert B.lib.rp_stage_upload_weights(None, 0, None, None, 0) == B.RP_EINVAL
    assert B.lib.rp_op_gemm(None, 9, 0, None, None, None, 1, 1, 8, 8, 8, 8, 1.0, 0, None, None, 0, 0, 0, None, 0, 0, None, 0) == B.RP_EINVAL
    assert B.lib.rp_op_rmsnorm_bwd_noalloc(None, None, 0, None, None, None, None, None, None, 8, 8) == B.RP_EINVAL


def test_workspace_covers_paper_activation_formula():
    """The per-layer internals kept by a backward stage are at least what App. B.1 (Eq. act-mem) counts."""
    from oracle import accounting
    c = synth.CONFIGS["C2"]
    cfg = H.cfg_from_dict(c)
    _, _, ws = B.rp_query_sizes(cfg, c["batch"], c["seq"])
    per_layer = accounting.activation_bytes_per_layer(c["seq"], c["batch"], c["hidden"], c["ffn"], c["n_q_heads"], c["n_kv_heads"])
    assert ws >= c["n_layers"] * per_layer
    assert ws <= 3.0 * c["n_layers"] * per_layer + 2 ** 31
