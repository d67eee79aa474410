"""A round of the multi-stream worker (paper Sec. 4.2): one stage over M micro-batches whose activations live in pinned
host memory, with the next stage's parameters streaming in and a finished stage's gradients streaming out inside the
round's transfer windows.  Checked through the C ABI against the CPU oracle (per micro-batch; weight gradients summed
over the micro-batches) and against the plain stage calls on device-resident activations."""
import numpy as np
import pytest

import parity_util as pu
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CFG = dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=344, vocab=0, n_experts=0, top_k=0,
           lora_rank=8, lora=("q", "v", "down"), train_base=1, batch=1, seq=264, x_from="normal")


@pytest.fixture(scope="module")
def hz():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_27085_amd import harness
    return harness


def pinned_bf16(hz, arr):
    t = torch.empty(arr.shape, dtype=torch.bfloat16, pin_memory=True)
    t.view(torch.int16).copy_(torch.from_numpy(hz.f32_to_bf16_bits(arr).view(np.int16).reshape(arr.shape)))
    return t


def tensor_mask(cfg, grads):
    """Boolean byte mask of the blob: True inside tensors, False in the alignment padding between chunks (which a round
    does not transfer: its items are the tensors)."""
    from paper_2604_27085_amd import binding as B
    wbytes, gbytes, _ = B.rp_query_sizes(cfg, 1, 8)
    mask = np.zeros(gbytes if grads else wbytes, dtype=bool)
    es = 4 if grads else 2
    for layer in range(cfg.n_layers + 1):
        for tid in range(len(B.TENSOR_IDS)):
            off, n = (B.rp_grad_layout if grads else B.rp_weight_layout)(cfg, layer, tid)
            mask[off:off + n * es] = True
    return mask


def draw_micro(c, seed, m):
    rng = np.random.default_rng(seed)
    T, h = c["batch"] * c["seq"], c["hidden"]
    xs = [synth.bf16_round(rng.standard_normal((T, h), dtype=np.float32)) for _ in range(m)]
    dys = [synth.bf16_round(rng.standard_normal((T, h), dtype=np.float32)) for _ in range(m)]
    return xs, dys


def test_forward_round_with_parameter_upload_matches_oracle(hz):
    """Three micro-batches through stage A while stage B's weights stream into the other slot in three windows (pieces
    of 64 KiB, so every large tensor is split); then one forward through B proves that the slot is complete."""
    from oracle import stage
    c, M = CFG, 3
    wlA = synth.make_workload(c, 2100, gains_random=True)
    wlB = synth.make_workload(c, 2101, gains_random=True)
    xs, _ = draw_micro(c, 2102, M)
    ocfg = pu.oracle_cfg(c)
    R = hz.StageRunner(hz.cfg_from_dict(c), c["batch"], c["seq"], n_slots=2)
    try:
        R.enable_rounds()
        hostA, hostB = R.pinned_blob(wlA["layers"]), R.pinned_blob(wlB["layers"])
        R.upload(hostA, slot=0)
        R.slots[1].fill_(0xFF)                      # NaN patterns: a missing piece would show
        x_host = [pinned_bf16(hz, x) for x in xs]
        out_host = [torch.zeros_like(t) for t in x_host]
        out_host = [t.pin_memory() for t in out_host]
        torch.cuda.synchronize()
        R.round(x_host, out_host, slot=0, next_slot=1, next_host_blob=hostB, max_piece_bytes=64 << 10)
        # stage B on the last output, straight after the round: must wait for its weights by itself
        xB = torch.empty_like(R.x_stage[0])
        R.sync()
        mask = tensor_mask(R.cfg, grads=False)
        assert mask.sum() > 0.99 * mask.size
        assert np.array_equal(R.slots[1][:R.wbytes].cpu().numpy()[mask], hostB.numpy()[mask])
        for j in range(M):
            ref, _ = stage.stage_fwd(xs[j].astype(np.float64), pu.cast_tree(wlA["layers"], np.float64), ocfg, c["batch"], c["seq"])
            got = out_host[j].float().numpy()
            assert pu.rel_l2(got, ref) <= 2e-2, (j, pu.rel_l2(got, ref))
            # identical to the plain call on a device-resident input (same kernels, same order)
            plain = R.forward(hz.bf16_tensor(xs[j], R.device), slot=0)
            R.sync()
            assert torch.equal(plain.cpu(), out_host[j])
        xB.copy_(out_host[M - 1])
        gotB = R.forward(xB, slot=1)
        R.sync()
        refB, _ = stage.stage_fwd(out_host[M - 1].float().numpy().astype(np.float64), pu.cast_tree(wlB["layers"], np.float64), ocfg,
                                  c["batch"], c["seq"])
        assert pu.rel_l2(hz.to_f32(gotB), refB) <= 2e-2
    finally:
        R.close()


@pytest.mark.parametrize("M", [1, 4])
def test_backward_round_with_gradient_download_matches_oracle(hz, M):
    """Backward rounds: input gradients per micro-batch, weight gradients accumulated over the M micro-batches, while a
    finished gradient blob goes home in the windows (bit-exact copy) and the next weights come in."""
    from oracle import stage
    c = CFG
    wl = synth.make_workload(c, 2200, gains_random=True)
    xs, dys = draw_micro(c, 2201 + M, M)
    ocfg = pu.oracle_cfg(c)
    layers64 = pu.cast_tree(wl["layers"], np.float64)
    cfg = hz.cfg_from_dict(c)
    R = hz.StageRunner(cfg, c["batch"], c["seq"], n_slots=2)
    try:
        R.enable_rounds()
        host = R.pinned_blob(wl["layers"])
        R.upload(host, slot=0)
        x_host = [pinned_bf16(hz, x) for x in xs]
        dy_host = [pinned_bf16(hz, d) for d in dys]
        dx_host = [torch.zeros_like(t).pin_memory() for t in x_host]
        done_dev = torch.randn(R.gbytes // 4, dtype=torch.float32, device=R.device)
        done_host = torch.zeros(R.gbytes // 4, dtype=torch.float32).pin_memory()
        torch.cuda.synchronize()
        R.round(x_host, dx_host, slot=0, dy_host=dy_host, next_slot=1, next_host_blob=host, done_grads_dev=done_dev,
                done_grads_host=done_host, max_piece_bytes=32 << 10)
        R.sync()
        gmask = tensor_mask(cfg, grads=True)
        assert np.array_equal(done_host.numpy().view(np.uint8)[gmask], done_dev.cpu().numpy().view(np.uint8)[gmask])
        wmask = tensor_mask(cfg, grads=False)
        assert np.array_equal(R.slots[1][:R.wbytes].cpu().numpy()[wmask], host.numpy()[wmask])
        want = None
        for j in range(M):
            _, dx, grads = stage.stage_fwd_bwd(xs[j].astype(np.float64), dys[j].astype(np.float64), layers64, ocfg, c["batch"], c["seq"])
            assert pu.rel_l2(dx_host[j].float().numpy(), dx) <= 2e-2, j
            if want is None:
                want = grads
            else:
                for li, g in enumerate(grads):
                    for k, v in g.items():
                        if k == "lora":
                            for nm, (dA, dB) in v.items():
                                a0, b0 = want[li]["lora"][nm]
                                want[li]["lora"][nm] = (a0 + dA, b0 + dB)
                        else:
                            want[li][k] = want[li][k] + v
        got_layers, _ = hz.unpack_grads(cfg, R.grads)
        errs = {}
        for li, g in enumerate(want):
            for k, v in g.items():
                if k == "lora":
                    for nm, (dA, dB) in v.items():
                        errs["L%d.%s.A" % (li, nm)] = pu.rel_l2(got_layers[li]["lora"][nm][0], dA)
                        errs["L%d.%s.B" % (li, nm)] = pu.rel_l2(got_layers[li]["lora"][nm][1], dB)
                else:
                    errs["L%d.%s" % (li, k)] = pu.rel_l2(got_layers[li][k], v)
        assert len(errs) == c["n_layers"] * (11 + 2 * len(c["lora"]))
        assert max(errs.values()) <= 2e-2, errs
    finally:
        R.close()


def test_round_error_paths(hz):
    from paper_2604_27085_amd import binding as B
    c = CFG
    R = hz.StageRunner(hz.cfg_from_dict(c), c["batch"], c["seq"], n_slots=2)
    try:
        wl = synth.make_workload(c, 2300)
        R.upload(R.pinned_blob(wl["layers"]), slot=0)
        x_host = [torch.zeros((R.T, c["hidden"]), dtype=torch.bfloat16).pin_memory()]
        out_host = [torch.zeros((R.T, c["hidden"]), dtype=torch.bfloat16).pin_memory()]
        stage_bufs = [torch.empty((R.T, c["hidden"]), dtype=torch.bfloat16, device=R.device) for _ in range(4)]
        io = B.make_round_io(x_host, out_host, stage_bufs[:2], stage_bufs[2:])
        with pytest.raises(B.RpError) as e:       # transfer streams not set
            B.rp_round_forward(R.ctx, 0, io, R.batch, R.seq, R.ws, R.wsbytes)
        assert e.value.code == B.RP_ESTATE
        R.enable_rounds()
        io = B.make_round_io(x_host, out_host, [stage_bufs[0], stage_bufs[0]], stage_bufs[2:])
        with pytest.raises(B.RpError) as e:       # both staging buffers the same
            B.rp_round_forward(R.ctx, 0, io, R.batch, R.seq, R.ws, R.wsbytes)
        assert e.value.code == B.RP_EINVAL
        io = B.make_round_io(x_host, out_host, stage_bufs[:2], stage_bufs[2:], next_slot=0, next_dev_slot=R.slots[0],
                             next_host_blob=x_host[0])
        with pytest.raises(B.RpError) as e:       # next slot is the slot being run
            B.rp_round_forward(R.ctx, 0, io, R.batch, R.seq, R.ws, R.wsbytes)
        assert e.value.code == B.RP_EINVAL
        R.sync()
    finally:
        R.close()
