"""End-to-end parity of the four hot-path calls (through the C ABI) against the CPU oracle: weight upload, forward
stage, backward stage with recomputation, LM head + cross-entropy.  Bounds: relative L2 error <= 2e-2 on every output
and gradient tensor, relative loss error <= 1e-4."""
import numpy as np
import pytest

import parity_util as pu
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def hz():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_27085_amd import harness
    return harness


def test_c1_chain_matches_oracle(hz):
    """Tiny stage: 2 layers + head, full fine-tune with LoRA on q and v, labels = next token."""
    c = synth.CONFIGS["C1"]
    wl = synth.make_workload(c, synth.config_seed("C1"))
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz)
    errs = pu.compare_chain(ref, got, c)
    # loss, head dx, head Wv/gf, out, dx, and per layer 11 base tensors + 4 adapter factors
    assert len(errs) == 4 + 2 + 2 * (11 + 4), sorted(errs)
    assert abs(ref["loss"] - np.log(c["vocab"])) < 0.5


def test_c1_fused_last_stage_matches_oracle_and_the_plain_calls(hz):
    """The fused last stage of Sec. 3.2 as bench.py times it -- forward keeping the internals, LM head on a workspace of
    its own, backward from the kept internals (rp_stage_backward with RP_PHASE_RECOMPUTE, then RP_PHASE_BACKWARD) --
    against the oracle, and bit for bit against forward stage -> head -> ordinary backward stage on the same inputs."""
    c = synth.CONFIGS["C1"]
    wl = synth.make_workload(c, synth.config_seed("C1"))
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz, fused=True)
    errs = pu.compare_chain(ref, got, c)
    assert len(errs) == 4 + 2 + 2 * (11 + 4), sorted(errs)
    plain = pu.gpu_chain(c, wl, hz)
    assert got["loss"] == plain["loss"]
    for k in ("out", "head_dx", "dx"):
        assert np.array_equal(got[k], plain[k]), k
    for k, v in plain["head_grads"].items():
        assert np.array_equal(got["head_grads"][k], v), k
    for gl, pl in zip(got["grads"], plain["grads"]):
        for k, v in pl.items():
            if k == "lora":
                for nm, (dA, dB) in v.items():
                    assert np.array_equal(gl["lora"][nm][0], dA) and np.array_equal(gl["lora"][nm][1], dB), nm
            elif v is not None:
                assert np.array_equal(gl[k], v), k


def test_backward_phase_alone_needs_the_router_logits_of_a_moe_stage(hz):
    """RP_PHASE_BACKWARD of a mixture-of-experts stage without router logits is an argument error, detected before
    anything is enqueued."""
    from paper_2604_27085_amd import binding as B
    c = MOE_VARIANTS["small"]
    cfg = hz.cfg_from_dict(c, with_head=False)
    R = hz.StageRunner(cfg, c["batch"], c["seq"])
    try:
        wl = synth.make_workload(c, 3)
        R.upload(R.pinned_blob(wl["layers"]))
        x = hz.bf16_tensor(wl["x"], R.device)
        dy = hz.bf16_tensor(wl["dy"], R.device)
        dx = torch.zeros_like(x)
        for phases in (B.PHASE_BACKWARD, B.PHASE_RECOMPUTE, B.PHASE_BOTH):
            with pytest.raises(B.RpError) as e:
                B.rp_stage_backward(R.ctx, 0, phases, x, dy, dx, None, R.grads, None, None, c["batch"], c["seq"], R.ws, R.wsbytes)
            assert e.value.code == B.RP_EINVAL
        with pytest.raises(B.RpError) as e:           # phases outside {1, 2, 3}
            B.rp_stage_backward(R.ctx, 0, 4, x, dy, dx, None, R.grads, None, None, c["batch"], c["seq"], R.ws, R.wsbytes)
        assert e.value.code == B.RP_EINVAL
        R.sync()
        assert float(dx.float().abs().sum()) == 0.0
    finally:
        R.close()


@pytest.mark.timeout(900)
def test_c2_full_size_every_stage_call_matches_oracle(hz, capsys):
    """The benchmark's workload at its full size and in the launch configuration bench.py times (Qwen3-1.7B-shaped
    layers, 4096 tokens, vocabulary 151936, 256x256 GEMM tiles, 32768-row vocabulary chunks).  Every call is checked
    against the oracle ON THE SAME INPUTS: the 4-layer forward produces the layer inputs, the head runs on the stage
    output the GPU produced, and each layer's backward stage (recomputation + backward, one layer per call) gets the
    GPU's own layer input and incoming gradient, so the bound applies to each call and not to a sum of their
    errors.  The oracle runs in fp32 here (its fp64 run takes minutes; fp32 rounding is three orders of magnitude
    below the bf16 bound)."""
    from oracle import stage

    def say(msg):                                  # a minute or two of work: say which part is running
        with capsys.disabled():
            print("[c2 full size] " + msg, flush=True)

    c = synth.CONFIGS["C2"]
    L, B_, S_ = c["n_layers"], c["batch"], c["seq"]
    say("generating the workload")
    wl = synth.make_workload(c, synth.config_seed("C2"))
    ocfg = pu.oracle_cfg(c)
    f32 = np.float32

    say("HIP path: 4-layer forward, head")
    cfg = hz.cfg_from_dict(c, with_head=True)
    R = hz.StageRunner(cfg, B_, S_)
    try:
        R.upload(R.pinned_blob(wl["layers"], wl["head"]))
        x = hz.bf16_tensor(wl["x"], R.device)
        labels = torch.from_numpy(wl["labels"]).to(R.device)
        torch.cuda.synchronize()
        out, keep = R.forward(x, keep_layer_inputs=True)
        loss, head_dx = R.head(out, labels, 1.0, train=True)
        R.sync()
        xs = [hz.to_f32(k) for k in keep]
        out_np, head_dx_np, loss_v = hz.to_f32(out), hz.to_f32(head_dx), float(loss.item())
        _, head_g = hz.unpack_grads(cfg, R.grads)
    finally:
        R.close()

    errs = {}
    say("oracle: head on the GPU's stage output")
    ref_loss, ref_dx, ref_hg = stage.head_fwd_bwd(out_np, pu.cast_tree(wl["head"], f32), wl["labels"], ocfg, 1.0, want_dW=True)
    errs["loss"] = abs(loss_v - float(ref_loss)) / abs(float(ref_loss))
    errs["head_dx"] = pu.rel_l2(head_dx_np, ref_dx)
    for k, v in ref_hg.items():
        errs["head." + k] = pu.rel_l2(head_g[k], v)
    del ref_dx, ref_hg, head_g

    c1 = dict(c, n_layers=1, vocab=0)
    cfg1 = hz.cfg_from_dict(c1, with_head=False)
    ocfg1 = pu.oracle_cfg(c1)
    dy_np = head_dx_np
    for l in reversed(range(L)):
        say("layer %d: HIP backward stage, oracle" % l)
        R1 = hz.StageRunner(cfg1, B_, S_)
        try:
            R1.upload(R1.pinned_blob([wl["layers"][l]]))
            xl, dyl = hz.bf16_tensor(xs[l], R1.device), hz.bf16_tensor(dy_np, R1.device)
            torch.cuda.synchronize()
            o_l, dx_l = R1.backward(xl, dyl)
            R1.sync()
            g_l, _ = hz.unpack_grads(cfg1, R1.grads)
            o_np, dx_np = hz.to_f32(o_l), hz.to_f32(dx_l)
        finally:
            R1.close()
        r_out, r_dx, r_g = stage.stage_fwd_bwd(xs[l], dy_np, [pu.cast_tree(wl["layers"][l], f32)], ocfg1, B_, S_)
        errs["L%d.out" % l] = pu.rel_l2(o_np, r_out)
        errs["L%d.dx" % l] = pu.rel_l2(dx_np, r_dx)
        for k, v in r_g[0].items():
            if k != "lora":
                errs["L%d.%s" % (l, k)] = pu.rel_l2(g_l[0][k], v)
        # the stage output of layer l must be the next layer's input (or the stage output) of the 4-layer call
        nxt = xs[l + 1] if l + 1 < L else out_np
        assert np.array_equal(o_np, nxt), "layer %d: single-layer and 4-layer calls disagree" % l
        dy_np = dx_np
    worst = max((v, k) for k, v in errs.items() if k != "loss")
    say("worst relative error %.2e (%s), loss error %.1e" % (worst + (errs["loss"],)))
    assert len(errs) == 4 + L * 13, sorted(errs)
    bad = {k: v for k, v in errs.items() if not v <= (1e-4 if k == "loss" else 2e-2)}
    assert not bad, "parity violations: %s\nall: %s" % (bad, errs)
    assert abs(loss_v - np.log(c["vocab"])) < 0.5


@pytest.mark.timeout(900)
def test_c2_full_size_fused_chain_against_the_never_rounding_oracle(hz, capsys):
    """The benchmark's workload at full size through the call sequence bench.py times (fused last stage: recompute ->
    head on its own workspace -> backward from the kept internals), compared AS ONE CHAIN with the oracle that never
    rounds: errors of four layers and the head accumulate.  Bound per tensor: 2e-2 wherever 16-bit storage allows it.
    On this workload it does not allow it everywhere: the residual stream is fed by an N(0, 0.02) embedding and is
    carried by the branch outputs alone, so every stored bf16 tensor's rounding reaches the next layers in full, and
    the attention backward multiplies what the forward left in q, k, v and the layer input (the gradients of Wq, Wk,
    gq, gk collect four such factors).  storage_rounding.bf16_storage() measures that floor with the oracle itself
    (its stored tensors rounded to bf16, nothing else changed, no HIP code involved); where the floor exceeds
    2e-2 / 1.25 the HIP path must stay within 25 % of the floor and below 3e-2 in any case.  Local bounds (single
    rows, blocks of 256 columns) apply with each tensor's bound."""
    from storage_rounding import bf16_storage

    def say(msg):
        with capsys.disabled():
            print("[c2 fused chain] " + msg, flush=True)

    c = synth.CONFIGS["C2"]
    say("generating the workload")
    wl = synth.make_workload(c, synth.config_seed("C2"))
    say("HIP path: fused last stage")
    got = pu.gpu_chain(c, wl, hz, fused=True)
    say("oracle (fp32), whole chain")
    ref = pu.oracle_chain(c, wl, dtype=np.float32)
    say("oracle with bf16 storage (the floor)")
    with bf16_storage():
        flo = pu.oracle_chain(c, wl, dtype=np.float32)
    floor = {n: pu.rel_l2(g, r) for n, g, r in pu.chain_pairs(ref, flo)}
    over = sorted(n for n, v in floor.items() if v > 2e-2)
    say("storage floor above 2e-2 on %d of %d tensors (%s), worst %.2e (%s)"
        % ((len(over), len(floor), " ".join(over)) + max((v, n) for n, v in floor.items())))
    assert all(n.split(".")[-1] in ("Wq", "Wk", "gq", "gk") for n in over), over      # the q/k path only
    tol_of = lambda n: min(3e-2, max(2e-2, 1.25 * floor[n]))
    errs = pu.compare_chain(ref, got, c, tol_of=tol_of)
    worst = max((v / tol_of(k), v, k) for k, v in errs.items() if k != "loss")
    say("worst tensor %.2e (%s) = %.2f of its bound; over the plain 2e-2: %s; loss error %.1e"
        % (worst[1], worst[2], worst[0], sorted(k for k, v in errs.items() if k != "loss" and v > 2e-2), errs["loss"]))
    assert len(errs) == 4 + 2 + c["n_layers"] * 11, sorted(errs)
    # everything off the q/k path meets the plain bound
    assert all(v <= 2e-2 for k, v in errs.items() if k != "loss" and k.split(".")[-1] not in ("Wq", "Wk", "gq", "gk"))


VARIANTS = {
    # ragged token count, every adapter on, frozen base, random gains
    "lora_all_frozen_ragged": dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=688, vocab=0,
                                   n_experts=0, top_k=0, lora_rank=16, lora=synth.LORA_ORDER, train_base=0, batch=1,
                                   seq=200, x_from="normal", lora_scale=2.0),
    # head_dim 128, two independent sequences, no QK-norm, full fine-tune without adapters
    "d128_batch2_nonorm": dict(n_layers=1, hidden=384, n_q_heads=2, n_kv_heads=1, head_dim=128, ffn=1024, vocab=0,
                               n_experts=0, top_k=0, lora_rank=0, lora=(), train_base=1, batch=2, seq=72,
                               x_from="normal", qk_norm=0),
    # adapters on k, o, gate only (partial fused groups), trainable base, group size 4
    "lora_partial_trainable": dict(n_layers=1, hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=64, ffn=768, vocab=0,
                                   n_experts=0, top_k=0, lora_rank=8, lora=("k", "o", "gate"), train_base=1, batch=1,
                                   seq=328, x_from="normal"),
}


MOE_VARIANTS = {
    # 8 experts, top-2, expert rows far below one 256-row tile; group size 2, LoRA on attention only, frozen base
    "small": dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=96, vocab=0, n_experts=8, top_k=2,
                  lora_rank=8, lora=("q", "k", "v", "o"), train_base=0, batch=1, seq=136, x_from="normal"),
    # more rows per expert than a tile (several tiles per expert, ragged tails), top-4 of 6, no adapters at all
    # the shape of C5 scaled down: 128 experts, top-8, head_dim 128 with 16 query heads per kv head, LoRA on attention
    "c5_like": dict(n_layers=1, hidden=256, n_q_heads=16, n_kv_heads=1, head_dim=128, ffn=96, vocab=0, n_experts=128,
                    top_k=8, lora_rank=8, lora=("q", "k", "v", "o"), train_base=0, batch=1, seq=1064, x_from="normal"),
    "tiles": dict(n_layers=1, hidden=128, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=64, vocab=0, n_experts=6, top_k=4,
                  lora_rank=0, lora=(), train_base=0, batch=2, seq=520, x_from="normal"),
}


@pytest.mark.parametrize("name", sorted(MOE_VARIANTS))
def test_moe_stage_matches_oracle(hz, name):
    """Top-k mixture-of-experts FFN: routing decisions are taken from the same fp32 logits on both sides, so they are
    identical; outputs, input gradient, router-logit gradients and adapter gradients within the bf16 bound."""
    c = MOE_VARIANTS[name]
    wl = synth.make_workload(c, 900 + sorted(MOE_VARIANTS).index(name), gains_random=True)
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz)
    errs = pu.compare_chain(ref, got, c)
    assert len(errs) == 2 + c["n_layers"] * (1 + 2 * len(c["lora"])), sorted(errs)
    # unselected experts get exactly zero gradient, selected ones do not
    for li in range(c["n_layers"]):
        assert np.array_equal(got["d_router"][li] == 0.0, ref["grads"][li]["router_logits"] == 0.0)


ROUTER_VARIANTS = {
    # the GPT-OSS-20B row scaled down: hidden and FFN width not multiples of the GEMM tiles (360 = 1.4 x 256), 4 of 32
    # experts, head_dim 64, eight query heads per kv head; two layers so that the second router sees a computed stream
    "oss_like": dict(n_layers=2, hidden=360, n_q_heads=8, n_kv_heads=1, head_dim=64, ffn=360, vocab=0, n_experts=32,
                     top_k=4, lora_rank=8, lora=("q", "k", "v", "o"), train_base=0, batch=1, seq=1032, x_from="normal",
                     moe_router=1),
    "e8": dict(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=96, vocab=0, n_experts=8, top_k=2,
               lora_rank=0, lora=(), train_base=0, batch=2, seq=136, x_from="normal", moe_router=1),
}


@pytest.mark.parametrize("name", sorted(ROUTER_VARIANTS))
def test_moe_router_in_stage_matches_oracle(hz, name):
    """Router weights in the layer: logits = n2 Wr^T computed by the stage, selection from them, and the gradient of the
    logits flowing back into n2.  The input has a planted, decisive preference per token, and the test first checks on
    the oracle's logits that every gap that decides the selection is far above the bf16 error of the logits -- then
    both sides must select the same experts, and everything is compared as for the other stages."""
    c = ROUTER_VARIANTS[name]
    seed = 1300 + sorted(ROUTER_VARIANTS).index(name)
    wl = synth.plant_routing(synth.make_workload(c, seed, gains_random=True), c, seed)
    ref = pu.oracle_chain(c, wl)
    k = c["top_k"]
    for lg in ref["logits"]:
        srt = -np.sort(-lg, axis=1)
        assert np.min(srt[:, k - 1] - srt[:, k]) > 0.05, "planted routing is not decisive"
    got = pu.gpu_chain(c, wl, hz)
    errs = pu.compare_chain(ref, got, c)
    assert len(errs) == 2 + c["n_layers"] * (2 + 2 * len(c["lora"])), sorted(errs)
    for li in range(c["n_layers"]):
        assert np.array_equal(got["d_router"][li] != 0.0, ref["grads"][li]["router_logits"] != 0.0)


def test_moe_router_in_stage_selection_is_topk_of_its_own_logits(hz):
    """Unstructured random router and input: near-ties exist, so the expert sets of the two sides may differ on a few
    tokens.  What is unique is checked -- the logits (floating point, within the bound) -- and the rest is checked for
    validity: the experts the stage selected (the non-zero pattern of the logit gradient) are exactly the top-k of the
    logits it reported, ties to the lower index, decided in the fp32 the kernel computes them in."""
    from oracle import layers as OL
    c = dict(ROUTER_VARIANTS["oss_like"], n_layers=1, seq=776)
    wl = synth.make_workload(c, 1400, gains_random=True)
    for p in wl["layers"]:
        p["Wr"] = synth.bf16_round(p["Wr"] * 3.0)        # logits of order one
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz)
    assert pu.rel_l2(got["logits"][0], ref["logits"][0]) <= 2e-2
    idx, _ = OL.moe_route(got["logits"][0], c["top_k"])
    sel = np.zeros_like(got["logits"][0], dtype=bool)
    np.put_along_axis(sel, idx, True, axis=1)
    assert np.array_equal(got["d_router"][0] != 0.0, sel)
    # tokens whose selection is decisive on the oracle's side agree with it
    srt = -np.sort(-ref["logits"][0], axis=1)
    decisive = (srt[:, c["top_k"] - 1] - srt[:, c["top_k"]]) > 0.05
    assert decisive.mean() > 0.5
    ref_sel = ref["grads"][0]["router_logits"] != 0.0
    assert np.array_equal(sel[decisive], ref_sel[decisive])
    assert pu.rel_l2(got["out"][decisive], ref["out"][decisive]) <= 2e-2
    # The gradient side.  The gradient of the logits is local to a token: on the decisive tokens it must match.
    assert pu.rel_l2(got["d_router"][0][decisive], ref["grads"][0]["router_logits"][decisive]) <= 2e-2
    # The input gradient and the adapter gradients mix all tokens through the attention backward, so they can only be
    # compared under one selection: the oracle is run again with its router's decision replaced, on the few tokens where
    # the two sides differ, by the (valid) decision the stage took -- its own logits, softmax over the forced picks --
    # and then everything is unique and compared in full.
    differ = np.nonzero((sel != ref_sel).any(axis=1))[0]
    assert 0 < len(differ) < 0.1 * sel.shape[0]          # near-ties exist on this input, and they are few
    orig_route = OL.moe_route

    def forced_route(logits, top_k):
        order, w = orig_route(logits, top_k)
        for t in differ:
            picks = np.nonzero(sel[t])[0]
            picks = picks[np.argsort(-logits[t, picks], kind="stable")]
            z = logits[t, picks] - logits[t, picks].max()
            order[t], w[t] = picks, np.exp(z) / np.exp(z).sum()
        return order, w

    OL.moe_route = forced_route
    try:
        ref2 = pu.oracle_chain(c, wl)
    finally:
        OL.moe_route = orig_route
    assert np.array_equal(ref2["grads"][0]["router_logits"] != 0.0, sel)
    errs = pu.compare_chain(ref2, got, c)
    assert len(errs) == 2 + 2 + 2 * len(c["lora"]), sorted(errs)


@pytest.mark.parametrize("name", sorted(VARIANTS))
def test_stage_variants_match_oracle(hz, name):
    c = VARIANTS[name]
    wl = synth.make_workload(c, 500 + sorted(VARIANTS).index(name), gains_random=True)
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz, use_upload=(name != "d128_batch2_nonorm"))
    errs = pu.compare_chain(ref, got, c)
    n_lora = 2 * len(c["lora"])
    n_base = (9 + (2 if c.get("qk_norm", 1) else 0)) if c["train_base"] else 0
    assert len(errs) == 2 + c["n_layers"] * (n_base + n_lora), sorted(errs)


def test_head_only_stage_ragged_vocab_and_ignored_rows(hz):
    """LM head as a stage of its own; vocabulary not a multiple of any tile, several vocabulary chunks are not needed
    here but the tail tile is; some rows ignored; loss scaling."""
    c = dict(n_layers=0, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=688, vocab=1000, n_experts=0, top_k=0,
             lora_rank=0, lora=(), train_base=1, batch=1, seq=136, x_from="normal")
    wl = synth.make_workload(c, 77, gains_random=True)
    wl["labels"][::5] = -100
    wl["x"] = synth.bf16_round(wl["x"] * 3.0)
    ref = pu.oracle_chain(c, wl, grad_scale=64.0)
    got = pu.gpu_chain(c, wl, hz, grad_scale=64.0)
    errs = pu.compare_chain(ref, got, c)
    assert set(errs) == {"loss", "head_dx", "head.Wv", "head.gf"}
    assert np.all(got["head_dx"][::5] == 0.0)


def test_frozen_head_reference_moves_between_chunks(hz):
    """Frozen head, one sweep over the vocabulary: the rows of later vocabulary chunks are scaled up so that their
    logits outgrow everything seen before by far more than the 2^8 the reference exponent tolerates -- the accumulated
    input gradient and normaliser must be rescaled; some labels ignored, some in the last (ragged) chunk, loss scaling."""
    c = dict(n_layers=0, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=256, vocab=40008, n_experts=0, top_k=0,
             lora_rank=0, lora=(), train_base=0, batch=1, seq=72, x_from="normal", head_chunk=16384)
    wl = synth.make_workload(c, 81, gains_random=True)
    Wv = wl["head"]["Wv"]
    Wv[16384:32768] *= 12.0          # second chunk: logits of order +-4 -> +-50
    Wv[32768:] *= 40.0               # third chunk larger still
    wl["head"]["Wv"] = synth.bf16_round(Wv)
    wl["labels"][::7] = -100
    wl["labels"][1::9] = 40007       # last row of the ragged last chunk
    wl["labels"][2::9] = 3           # first chunk: its logit is tiny against the later ones
    ref = pu.oracle_chain(c, wl, grad_scale=32.0)
    got = pu.gpu_chain(c, wl, hz, grad_scale=32.0)
    errs = pu.compare_chain(ref, got, c)
    assert set(errs) == {"loss", "head_dx"}
    ignored = wl["labels"] == -100
    assert ignored.sum() >= 8 and np.all(got["head_dx"][ignored] == 0.0)
    assert ref["loss"] > 20.0        # the loss is dominated by the large logits: the rescale path was exercised


def test_trainable_head_in_one_sweep_when_the_reference_moves_between_chunks(hz):
    """Trainable head, one sweep: the probabilities of every chunk stay in memory against the reference exponent and the
    weight gradient is formed from them afterwards.  As above, later chunks outgrow the earlier ones -- the second by
    less than the limit (probabilities of order e^44 are stored as they are), the third by more (the reference moves:
    the accumulated input gradient, the normaliser AND the probabilities already stored are rescaled).  dW rows of all
    three chunks, the final norm's gain gradient, dx and the loss against the oracle; labels in every chunk, some
    ignored; and the two-sweep schedule (cfg.head_two_sweeps) gives the same within the bf16 noise."""
    c = dict(n_layers=0, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=256, vocab=40008, n_experts=0, top_k=0,
             lora_rank=0, lora=(), train_base=1, batch=1, seq=72, x_from="normal", head_chunk=16384)
    wl = synth.make_workload(c, 82, gains_random=True)
    Wv = wl["head"]["Wv"]
    Wv[16384:32768] *= 12.0
    Wv[32768:] *= 40.0
    wl["head"]["Wv"] = synth.bf16_round(Wv)
    wl["labels"][::7] = -100
    wl["labels"][1::9] = 40007       # last row of the ragged last chunk
    wl["labels"][2::9] = 3           # first chunk
    wl["labels"][3::9] = 20000       # second chunk
    ref = pu.oracle_chain(c, wl, grad_scale=32.0)
    got = pu.gpu_chain(c, wl, hz, grad_scale=32.0)
    errs = pu.compare_chain(ref, got, c)
    assert {"loss", "head_dx", "head.Wv", "head.gf"} <= set(errs), sorted(errs)
    assert ref["loss"] > 20.0
    # rows of the first chunk receive gradient only through probabilities that were rescaled twice; they must not be lost
    gw, rw = got["head_grads"]["Wv"], ref["head_grads"]["Wv"]
    for lo, hi in ((0, 16384), (16384, 32768), (32768, 40008)):
        assert pu.rel_l2(gw[lo:hi], rw[lo:hi]) < 2e-2, (lo, hi)
    two = pu.gpu_chain(dict(c, head_two_sweeps=1), wl, hz, grad_scale=32.0)
    assert pu.rel_l2(two["head_grads"]["Wv"], gw) < 1e-2 and pu.rel_l2(two["head_dx"], got["head_dx"]) < 1e-2
    assert abs(two["loss"] - got["loss"]) <= 1e-5 * abs(got["loss"])


def test_frozen_head_single_ragged_chunk(hz):
    """Frozen head whose vocabulary fits one chunk and is not a multiple of any tile; ragged token count."""
    c = dict(n_layers=0, hidden=128, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=256, vocab=1000, n_experts=0, top_k=0,
             lora_rank=0, lora=(), train_base=0, batch=1, seq=136, x_from="normal")
    wl = synth.make_workload(c, 83, gains_random=True)
    wl["x"] = synth.bf16_round(wl["x"] * 4.0)
    wl["labels"][5::11] = -100
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz)
    errs = pu.compare_chain(ref, got, c)
    assert set(errs) == {"loss", "head_dx"}


def test_head_multiple_vocab_chunks_frozen(hz):
    """Vocabulary larger than one chunk (32768 rows at this token count) with a frozen head: only loss and dx."""
    c = dict(n_layers=0, hidden=128, n_q_heads=2, n_kv_heads=1, head_dim=64, ffn=256, vocab=40000, n_experts=0, top_k=0,
             lora_rank=0, lora=(), train_base=0, batch=1, seq=64, x_from="normal")
    wl = synth.make_workload(c, 78)
    ref = pu.oracle_chain(c, wl)
    got = pu.gpu_chain(c, wl, hz)
    errs = pu.compare_chain(ref, got, c)
    assert set(errs) == {"loss", "head_dx"}


def test_gradients_accumulate_over_micro_batches(hz):
    c = VARIANTS["lora_partial_trainable"]
    wl = synth.make_workload(c, 9)
    cfg = hz.cfg_from_dict(c, with_head=False)
    R = hz.StageRunner(cfg, c["batch"], c["seq"])
    try:
        R.upload(R.pinned_blob(wl["layers"]))
        x, dy = hz.bf16_tensor(wl["x"], R.device), hz.bf16_tensor(wl["dy"], R.device)
        torch.cuda.synchronize()
        _, dx1 = R.backward(x, dy)
        R.sync()
        g1 = R.grads.clone()
        _, dx2 = R.backward(x, dy)
        R.sync()
        assert torch.equal(dx1, dx2)
        l1, _ = hz.unpack_grads(cfg, g1)
        l2, _ = hz.unpack_grads(cfg, R.grads)
        # every weight gradient is summed in a fixed order (reduction splits merge through scratch memory in slice order,
        # gain gradients through per-block partials): the second pass doubles the first exactly
        for k, v in l1[0].items():
            if k == "lora":
                for nm, (dA, dB) in v.items():
                    np.testing.assert_array_equal(l2[0]["lora"][nm][0], 2 * dA, err_msg=nm)
                    np.testing.assert_array_equal(l2[0]["lora"][nm][1], 2 * dB, err_msg=nm)
            elif v is not None:
                np.testing.assert_array_equal(l2[0][k], 2 * v, err_msg=k)
    finally:
        R.close()


def test_forward_stage_checkpoints_and_matches_backward_recompute(hz):
    from oracle import stage
    c = synth.CONFIGS["C1"]
    wl = synth.make_workload(c, 11)
    cfg = hz.cfg_from_dict(c, with_head=False)
    R = hz.StageRunner(cfg, c["batch"], c["seq"])
    try:
        R.upload(R.pinned_blob(wl["layers"]))
        x = hz.bf16_tensor(wl["x"], R.device)
        dy = hz.bf16_tensor(wl["dy"], R.device)
        torch.cuda.synchronize()
        out, keep = R.forward(x, keep_layer_inputs=True)
        out_b, _ = R.backward(x, dy)
        R.sync()
        assert torch.equal(out, out_b)                 # the recomputation reproduces the forward stage bit for bit
        assert torch.equal(keep[0], x)
        ocfg = pu.oracle_cfg(dict(c, vocab=0))
        ref_out, ref_inputs = stage.stage_fwd(wl["x"].astype(np.float64), pu.cast_tree(wl["layers"], np.float64), ocfg,
                                              c["batch"], c["seq"])
        assert pu.rel_l2(hz.to_f32(out), ref_out) < 2e-2
        assert pu.rel_l2(hz.to_f32(keep[1]), ref_inputs[1]) < 2e-2
    finally:
        R.close()


def test_error_paths_leave_no_work_enqueued(hz):
    from paper_2604_27085_amd import binding as B
    c = synth.CONFIGS["C1"]
    cfg = hz.cfg_from_dict(c)
    R = hz.StageRunner(cfg, c["batch"], c["seq"])
    try:
        x = torch.zeros((R.T, c["hidden"]), dtype=torch.bfloat16, device=R.device)
        y = torch.zeros_like(x)
        with pytest.raises(B.RpError) as e:           # nothing uploaded yet
            B.rp_stage_forward(R.ctx, 0, x, y, None, None, c["batch"], c["seq"], R.ws, R.wsbytes)
        assert e.value.code == B.RP_ESTATE
        wl = synth.make_workload(c, 1)
        host = R.pinned_blob(wl["layers"], wl["head"])
        with pytest.raises(B.RpError) as e:
            B.rp_stage_upload_weights(R.ctx, 0, R.slots[0], host, R.wbytes - 256)
        assert e.value.code == B.RP_EINVAL
        R.upload(host)
        with pytest.raises(B.RpError) as e:
            B.rp_stage_forward(R.ctx, 0, x, y, None, None, c["batch"], c["seq"], R.ws, 1024)
        assert e.value.code == B.RP_ENOMEM
        with pytest.raises(B.RpError) as e:
            B.rp_stage_forward(R.ctx, 0, x, x, None, None, c["batch"], c["seq"], R.ws, R.wsbytes)
        assert e.value.code == B.RP_EINVAL
        with pytest.raises(B.RpError) as e:
            B.rp_stage_forward(R.ctx, 9, x, y, None, None, c["batch"], c["seq"], R.ws, R.wsbytes)
        assert e.value.code == B.RP_EINVAL
        R.sync()
        assert float(y.float().abs().sum()) == 0.0
    finally:
        R.close()


def test_upload_event_gating_against_poisoned_slot(hz):
    """The slot is filled with NaN bit patterns on the compute stream right before the upload; the stage must wait for
    each layer's bytes (per-layer events), so no NaN may reach the output."""
    c = synth.CONFIGS["C1"]
    wl = synth.make_workload(c, 21)
    cfg = hz.cfg_from_dict(c, with_head=False)
    R = hz.StageRunner(cfg, c["batch"], c["seq"], n_slots=2)
    try:
        host = R.pinned_blob(wl["layers"])
        x = hz.bf16_tensor(wl["x"], R.device)
        for s in range(2):
            R.slots[s].fill_(0xFF)
        torch.cuda.synchronize()
        outs = []
        for step in range(4):
            s = step & 1
            R.upload(host, slot=s)
            outs.append(R.forward(x, slot=s))
        R.sync()
        for o in outs:
            assert torch.isfinite(o.float()).all()
            assert torch.equal(o, outs[0])
    finally:
        R.close()
