"""Checks at the FULL sequence lengths of the larger workloads (16384 tokens with 64/8 heads, 31744 tokens with 64/4
heads and 128 experts), where the CPU oracle cannot run the whole problem: closed forms that do not use the oracle's
formula, single rows and key positions computed one by one from the plain definition, and properties that hold at any
size.  They reach the code paths only these sizes reach: operands of 0.5-2 GB addressed with 32-bit byte offsets, tens
of thousands of workgroups per attention launch, 253952 expert-sorted rows in the grouped products."""
import numpy as np
import pytest

import parity_util as pu
import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SHAPES = {"c4_length": (16384, 64, 8), "c5_length": (31744, 64, 4)}      # seq, query heads, kv heads; head_dim 128
D = 128


@pytest.fixture(scope="module")
def rp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_27085_amd import binding, harness
    return binding, harness


def stream():
    return torch.cuda.current_stream().cuda_stream


def rel(a, b):
    return pu.rel_l2(a, b)


def run_attention(B, H, q, k, v, do, seq, a, kh, batch=1, D=D):
    """q, do: bf16 device [T, a*D]; k, v: [T, kh*D], T = batch * seq.  Returns o, lse, dq, dk, dv as float32 ndarrays
    ([seq, heads, D] and lse [a, seq]; with batch > 1 a leading batch axis)."""
    dv_ = "cuda:0"
    o = torch.empty_like(q)
    lse = torch.empty((batch, a, seq), dtype=torch.float32, device=dv_)
    B.rp_op_attn_fwd(stream(), q, k, v, o, lse, a * D, kh * D, kh * D, a * D, batch, seq, a, kh, D)
    dq = torch.empty_like(q)
    dk, dvv = torch.empty_like(k), torch.empty_like(v)
    delta = torch.empty((batch, a, seq), dtype=torch.float32, device=dv_)
    scratch = torch.empty((2, batch * seq, a * D), dtype=torch.float32, device=dv_)
    B.rp_op_attn_bwd(stream(), q, k, v, o, do, lse, delta, dq, dk, dvv, scratch, a * D, kh * D, kh * D, a * D, a * D, a * D,
                     kh * D, kh * D, batch, seq, a, kh, D)
    torch.cuda.synchronize()
    if batch == 1:
        f = lambda t, h: H.to_f32(t).reshape(seq, h, D)
        return f(o, a), lse.cpu().numpy()[0], f(dq, a), f(dk, kh), f(dvv, kh)
    f = lambda t, h: H.to_f32(t).reshape(batch, seq, h, D)
    return f(o, a), lse.cpu().numpy(), f(dq, a), f(dk, kh), f(dvv, kh)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", sorted(SHAPES))
def test_zero_queries_give_running_means_at_full_length(rp, name, capsys):
    """q = 0: every score is 0, so row t of the softmax is uniform over keys 0..t.  Closed forms over the WHOLE tensors:
    o_t = mean(v_0..t), lse_t = ln(t+1); backward: dv_s = sum over the group's heads and t >= s of dO_t / (t+1), dk = 0
    (it is proportional to q), and on sampled rows dq_t = (dO_t (V_<=t - o_t)^T) K_<=t / ((t+1) sqrt(d))."""
    B, H = rp
    seq, a, kh = SHAPES[name]
    grp = a // kh
    with capsys.disabled():
        print("[%s] zero queries, seq %d, %d/%d heads" % (name, seq, a, kh), flush=True)
    rng = np.random.default_rng(seq)
    k = synth.bf16_round(rng.standard_normal((seq, kh, D), dtype=np.float32))
    v = synth.bf16_round(rng.standard_normal((seq, kh, D), dtype=np.float32))
    do = synth.bf16_round(rng.standard_normal((seq, a, D), dtype=np.float32))
    qd = torch.zeros((seq, a * D), dtype=torch.bfloat16, device="cuda:0")
    o, lse, dq, dk, dv = run_attention(B, H, qd, H.bf16_tensor(k.reshape(seq, -1), "cuda:0"), H.bf16_tensor(v.reshape(seq, -1), "cuda:0"),
                                       H.bf16_tensor(do.reshape(seq, -1), "cuda:0"), seq, a, kh)
    cnt = np.arange(1, seq + 1, dtype=np.float64)
    mean_v = np.cumsum(v.astype(np.float64), axis=0) / cnt[:, None, None]                 # [seq, kh, D]
    assert np.max(np.abs(lse - np.log(cnt)[None, :])) < 2e-5
    worst = max(rel(o[:, j], mean_v[:, j // grp]) for j in range(a))
    assert worst < 4e-3, worst
    # per-row check as well: the last rows average 16384 / 31744 values and are the smallest
    for j in (0, a - 1):
        err = np.linalg.norm(o[:, j] - mean_v[:, j // grp], axis=1) / np.linalg.norm(mean_v[:, j // grp], axis=1)
        assert err.max() < 2e-2, (j, int(err.argmax()), err.max())
    w = do.astype(np.float64) / cnt[:, None, None]                                          # dO_t / (t+1)
    rev = np.cumsum(w[::-1], axis=0)[::-1]                                                  # sum over t >= s
    dv_ref = rev.reshape(seq, kh, grp, D).sum(axis=2)
    assert rel(dv, dv_ref) < 6e-3
    err = np.linalg.norm((dv - dv_ref).reshape(seq, -1), axis=1) / np.linalg.norm(dv_ref.reshape(seq, -1), axis=1)
    assert err.max() < 3e-2, (int(err.argmax()), err.max())
    assert np.max(np.abs(dk)) <= 1e-6 * np.max(np.abs(dv))
    k64, v64 = k.astype(np.float64), v.astype(np.float64)
    for t in (0, 1, 63, 64, 127, 128, 4095, 4096, seq // 2 + 17, seq - 129, seq - 128, seq - 1):
        for j in (0, grp - 1, grp, a - 1):
            g = j // grp
            dp = v64[: t + 1, g] @ do[t, j].astype(np.float64) - mean_v[t, g] @ do[t, j].astype(np.float64)
            ref = (dp @ k64[: t + 1, g]) / ((t + 1) * np.sqrt(D))
            assert np.linalg.norm(dq[t, j] - ref) <= 1.5e-2 * np.linalg.norm(ref) + 5e-5, (t, j)      # t = 0: exactly zero


@pytest.mark.timeout(600)
def test_zero_queries_two_sequences_of_ragged_length(rp, capsys):
    """The same closed forms for a batch of two sequences whose length (12424) is a multiple of none of the tile sizes:
    98 key tiles of 128 put the dK/dV kernel on its XCD-aware launch order with a ragged last run (positions past the
    last key tile exit), 16/4 heads x 2 sequences give every XCD four heads, and the forward and dQ kernels run their
    256-query workgroups with a ragged last one.  Different values per sequence: a kernel that mixed the two up, or
    dropped a tile of either, would miss the running means."""
    B, H = rp
    batch, seq, a, kh = 2, 12424, 16, 4
    grp = a // kh
    with capsys.disabled():
        print("[batch 2] zero queries, seq %d, %d/%d heads" % (seq, a, kh), flush=True)
    rng = np.random.default_rng(77)
    k = synth.bf16_round(rng.standard_normal((batch, seq, kh, D), dtype=np.float32))
    v = synth.bf16_round(rng.standard_normal((batch, seq, kh, D), dtype=np.float32))
    do = synth.bf16_round(rng.standard_normal((batch, seq, a, D), dtype=np.float32))
    qd = torch.zeros((batch * seq, a * D), dtype=torch.bfloat16, device="cuda:0")
    dev = lambda t: H.bf16_tensor(t.reshape(batch * seq, -1), "cuda:0")
    o, lse, dq, dk, dv = run_attention(B, H, qd, dev(k), dev(v), dev(do), seq, a, kh, batch)
    cnt = np.arange(1, seq + 1, dtype=np.float64)
    for b in range(batch):
        mean_v = np.cumsum(v[b].astype(np.float64), axis=0) / cnt[:, None, None]
        assert np.max(np.abs(lse[b] - np.log(cnt)[None, :])) < 2e-5
        for j in range(a):
            err = np.linalg.norm(o[b, :, j] - mean_v[:, j // grp], axis=1) / np.linalg.norm(mean_v[:, j // grp], axis=1)
            assert rel(o[b, :, j], mean_v[:, j // grp]) < 4e-3 and err.max() < 2e-2, (b, j, int(err.argmax()), err.max())
        w = do[b].astype(np.float64) / cnt[:, None, None]
        dv_ref = np.cumsum(w[::-1], axis=0)[::-1].reshape(seq, kh, grp, D).sum(axis=2)
        assert rel(dv[b], dv_ref) < 6e-3
        err = np.linalg.norm((dv[b] - dv_ref).reshape(seq, -1), axis=1) / np.linalg.norm(dv_ref.reshape(seq, -1), axis=1)
        assert err.max() < 3e-2, (b, int(err.argmax()), err.max())
        assert np.max(np.abs(dk[b])) <= 1e-6 * np.max(np.abs(dv[b]))
        k64, v64 = k[b].astype(np.float64), v[b].astype(np.float64)
        for t in (0, 127, 128, 6000, seq - 129, seq - 9, seq - 1):
            for j in (0, grp, a - 1):
                g = j // grp
                dp = v64[: t + 1, g] @ do[b, t, j].astype(np.float64) - mean_v[t, g] @ do[b, t, j].astype(np.float64)
                ref = (dp @ k64[: t + 1, g]) / ((t + 1) * np.sqrt(D))
                assert np.linalg.norm(dq[b, t, j] - ref) <= 1.5e-2 * np.linalg.norm(ref) + 5e-5, (b, t, j)


@pytest.mark.timeout(600)
def test_zero_queries_head_dim_64_at_ragged_length(rp, capsys):
    """Head dimension 64 (the GPT-OSS shape) at 12424 tokens with 32/8 heads: long enough for the XCD-aware order of the
    dK/dV kernel (98 key tiles, ragged last run) and for thousands of workgroups per launch, which the short kernel tests
    do not reach at this head dimension.  Same closed forms as above."""
    B, H = rp
    seq, a, kh, d = 12424, 32, 8, 64
    grp = a // kh
    with capsys.disabled():
        print("[d = 64] zero queries, seq %d, %d/%d heads" % (seq, a, kh), flush=True)
    rng = np.random.default_rng(64)
    k = synth.bf16_round(rng.standard_normal((seq, kh, d), dtype=np.float32))
    v = synth.bf16_round(rng.standard_normal((seq, kh, d), dtype=np.float32))
    do = synth.bf16_round(rng.standard_normal((seq, a, d), dtype=np.float32))
    qd = torch.zeros((seq, a * d), dtype=torch.bfloat16, device="cuda:0")
    dev = lambda t: H.bf16_tensor(t.reshape(seq, -1), "cuda:0")
    o, lse, dq, dk, dv = run_attention(B, H, qd, dev(k), dev(v), dev(do), seq, a, kh, 1, d)
    cnt = np.arange(1, seq + 1, dtype=np.float64)
    mean_v = np.cumsum(v.astype(np.float64), axis=0) / cnt[:, None, None]
    assert np.max(np.abs(lse - np.log(cnt)[None, :])) < 2e-5
    for j in range(a):
        err = np.linalg.norm(o[:, j] - mean_v[:, j // grp], axis=1) / np.linalg.norm(mean_v[:, j // grp], axis=1)
        assert rel(o[:, j], mean_v[:, j // grp]) < 4e-3 and err.max() < 2e-2, (j, int(err.argmax()), err.max())
    w = do.astype(np.float64) / cnt[:, None, None]
    dv_ref = np.cumsum(w[::-1], axis=0)[::-1].reshape(seq, kh, grp, d).sum(axis=2)
    assert rel(dv, dv_ref) < 6e-3
    err = np.linalg.norm((dv - dv_ref).reshape(seq, -1), axis=1) / np.linalg.norm(dv_ref.reshape(seq, -1), axis=1)
    assert err.max() < 3e-2, (int(err.argmax()), err.max())
    assert np.max(np.abs(dk)) <= 1e-6 * np.max(np.abs(dv))
    k64, v64 = k.astype(np.float64), v.astype(np.float64)
    for t in (0, 63, 64, 255, 256, 6000, seq - 129, seq - 9, seq - 1):
        for j in (0, grp, a - 1):
            g = j // grp
            dp = v64[: t + 1, g] @ do[t, j].astype(np.float64) - mean_v[t, g] @ do[t, j].astype(np.float64)
            ref = (dp @ k64[: t + 1, g]) / ((t + 1) * np.sqrt(d))
            assert np.linalg.norm(dq[t, j] - ref) <= 1.5e-2 * np.linalg.norm(ref) + 5e-5, (t, j)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", sorted(SHAPES))
def test_sampled_rows_and_late_keys_match_the_definition_at_full_length(rp, name, capsys):
    """Random q, k, v, dO at the full shape.  Single query rows (first and last tiles, tile edges, the middle) are
    computed from the definition: o_t, lse_t and dq_t depend on row t alone.  dk_s and dv_s of the last 128 keys depend
    on the few query rows t >= s, which are computed in full for every head of the key's group.  Properties of the
    whole tensors: the keys' dv sum to the sum of dO over the group (softmax rows sum to 1) and their dk sum to zero
    (rows of dS sum to 0)."""
    B, H = rp
    seq, a, kh = SHAPES[name]
    grp = a // kh
    with capsys.disabled():
        print("[%s] sampled rows, seq %d, %d/%d heads" % (name, seq, a, kh), flush=True)
    rng = np.random.default_rng(seq + 1)
    draw = lambda h: synth.bf16_round(rng.standard_normal((seq, h, D), dtype=np.float32))
    q, k, v, do = draw(a), draw(kh), draw(kh), draw(a)
    dev = lambda t: H.bf16_tensor(t.reshape(seq, -1), "cuda:0")
    o, lse, dq, dk, dv = run_attention(B, H, dev(q), dev(k), dev(v), dev(do), seq, a, kh)
    sc = 1.0 / np.sqrt(D)
    k64 = np.ascontiguousarray(k.astype(np.float64).transpose(1, 0, 2))      # [kh, seq, D]
    v64 = np.ascontiguousarray(v.astype(np.float64).transpose(1, 0, 2))

    def row(t, j):      # the definition, restricted to query row t of head j (float64)
        g = j // grp
        kk, vv, dot = k64[g, : t + 1], v64[g, : t + 1], do[t, j].astype(np.float64)
        s = (kk @ q[t, j].astype(np.float64)) * sc
        m = s.max()
        e = np.exp(s - m)
        l = e.sum()
        p = e / l
        o_t = p @ vv
        ds = p * (vv @ dot - dot @ o_t)
        return o_t, m + np.log(l), (ds @ kk) * sc, p, ds

    for t in (0, 5, 31, 32, 127, 128, 129, 8191, 8192, seq // 2 + 77, seq - 257, seq - 128, seq - 65, seq - 1):
        for j in (0, 1, grp - 1, grp, a - grp, a - 1):
            o_t, lse_t, dq_t, _, _ = row(t, j)
            assert np.linalg.norm(o[t, j] - o_t) <= 1e-2 * np.linalg.norm(o_t), (t, j)
            assert abs(lse[j, t] - lse_t) < 2e-3, (t, j)
            assert np.linalg.norm(dq[t, j] - dq_t) <= 2e-2 * np.linalg.norm(dq_t) + 5e-5, (t, j)     # t = 0: exactly zero
    # the last 128 keys of the first and the last kv head: all query rows that see them, all heads of the group
    n_late = 128
    for g in (0, kh - 1):
        dk_ref = np.zeros((n_late, D))
        dv_ref = np.zeros((n_late, D))
        for j in range(g * grp, (g + 1) * grp):
            for t in range(seq - n_late, seq):
                _, _, _, p, ds = row(t, j)
                lo = seq - n_late
                dv_ref[: t + 1 - lo] += np.outer(p[lo:], do[t, j].astype(np.float64))
                dk_ref[: t + 1 - lo] += np.outer(ds[lo:], q[t, j].astype(np.float64)) * sc
        assert rel(dv[seq - n_late:, g], dv_ref) < 1e-2, g
        assert rel(dk[seq - n_late:, g], dk_ref) < 1.5e-2, g
    # whole-tensor properties
    sum_do = do.astype(np.float64).reshape(seq, kh, grp, D).sum(axis=(0, 2))
    sum_dv = dv.astype(np.float64).sum(axis=0)
    assert rel(sum_dv, sum_do) < 5e-3
    sum_dk = np.abs(dk.astype(np.float64).sum(axis=0)).max()
    assert sum_dk < 2e-3 * np.abs(dk).sum(axis=0).max(), sum_dk


@pytest.mark.timeout(600)
def test_zero_input_head_has_loss_ln_v_at_full_length(rp, capsys):
    """x = 0 at 16384 tokens, hidden 5120, vocabulary 151936 (the frozen head of the 32B-shaped workload, one sweep,
    16384-row chunks): the normalised input is 0, every logit is 0, so loss = ln V exactly; the gradient of the logits is
    (1/V - onehot) / N_valid and the RMSNorm backward at x = 0 reduces to a scale by g / sqrt(eps):
    dx_t = g * (mean_v W_v - W[y_t]) / (N_valid sqrt(eps))."""
    B, H = rp
    c = dict(synth.CONFIGS["C4"], n_layers=0, lora_rank=0, lora=())
    T, h, V = c["seq"], c["hidden"], c["vocab"]
    with capsys.disabled():
        print("[c4 head] zero input, %d tokens, vocabulary %d" % (T, V), flush=True)
    rng = np.random.default_rng(404)
    head = synth.make_head(rng, c, gains_random=True)
    labels = rng.integers(0, V, size=T).astype(np.int32)
    labels[::9] = -100
    labels[1] = V - 1
    cfg = H.cfg_from_dict(c, with_head=True)
    R = H.StageRunner(cfg, 1, T)
    try:
        R.upload(R.pinned_blob([], head))
        x = torch.zeros((T, h), dtype=torch.bfloat16, device=R.device)
        loss, dx = R.head(x, torch.from_numpy(labels).to(R.device), 1.0, train=False)
        R.sync()
        loss_v, dx = float(loss.item()), H.to_f32(dx)
    finally:
        R.close()
    assert abs(loss_v - np.log(V)) < 1e-5 * np.log(V)
    valid = labels != -100
    W = head["Wv"].astype(np.float64)
    ref = (W.mean(axis=0)[None, :] - W[labels[valid]]) * head["gf"].astype(np.float64)[None, :] / (valid.sum() * np.sqrt(c.get("rms_eps", 1e-6)))
    assert np.all(dx[~valid] == 0.0)
    assert rel(dx[valid], ref) < 4e-3
    err = np.linalg.norm(dx[valid] - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert err.max() < 1e-2, err.max()


@pytest.mark.timeout(900)
def test_identical_experts_reduce_the_moe_layer_to_the_dense_one_at_full_length(rp, capsys):
    """31744 tokens, 128 experts, top-8, hidden 4096, expert width 1536, 64/4 heads: when every expert holds the same
    weights the routing weights (which sum to 1) drop out and the layer is the dense layer with that FFN -- forward,
    input gradient and adapter gradients -- whatever the router logits are; the gradient of the logits vanishes (every
    expert's dw is the same).  The dense stage is the reference (its kernels are checked against the oracle at this
    width); the mixture runs its routing, counting sort over 253952 rows and grouped products at full size."""
    B, H = rp
    c = synth.CONFIGS["C5"]
    T = c["seq"]
    with capsys.disabled():
        print("[c5 moe] identical experts, %d tokens, %d experts, top-%d" % (T, c["n_experts"], c["top_k"]), flush=True)
    dense = dict(c, n_experts=0, top_k=0)
    wl = synth.make_workload(dense, 505, gains_random=True)           # one dense layer: Wg, Wu [m, h], Wd [h, m]
    rng = np.random.default_rng(506)
    logits = rng.standard_normal((1, T, c["n_experts"]), dtype=np.float32)

    def run(cc, layers, router):
        cfg = H.cfg_from_dict(cc, with_head=False)
        R = H.StageRunner(cfg, 1, T)
        try:
            R.upload(R.pinned_blob(layers))
            x, dy = H.bf16_tensor(wl["x"], R.device), H.bf16_tensor(wl["dy"], R.device)
            r = torch.from_numpy(router).to(R.device) if router is not None else None
            dr = torch.full_like(r, float("nan")) if r is not None else None
            out, dx = R.backward(x, dy, router=r, d_router=dr)
            R.sync()
            g, _ = H.unpack_grads(cfg, R.grads)
            return H.to_f32(out), H.to_f32(dx), g[0]["lora"], (dr.cpu().numpy() if dr is not None else None)
        finally:
            R.close()

    p = wl["layers"][0]
    E = c["n_experts"]
    moe_layer = dict(p, Wg=np.broadcast_to(p["Wg"], (E,) + p["Wg"].shape), Wu=np.broadcast_to(p["Wu"], (E,) + p["Wu"].shape),
                     Wd=np.broadcast_to(p["Wd"], (E,) + p["Wd"].shape))
    out_m, dx_m, lora_m, dlog = run(c, [moe_layer], logits)
    out_d, dx_d, lora_d, _ = run(dense, [p], None)
    # two bf16 pipelines that round at different points: each is within ~4e-3 of the exact layer
    assert rel(out_m, out_d) < 8e-3
    assert rel(dx_m, dx_d) < 1.2e-2
    for nm in c["lora"]:
        for i in (0, 1):
            assert rel(lora_m[nm][i], lora_d[nm][i]) < 1.5e-2, (nm, i)
    for got, ref in ((out_m, out_d), (dx_m, dx_d)):       # no dead row in 31744
        err = np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)
        assert err.max() < 6e-2, (int(err.argmax()), err.max())
    # d logits = w (dw - sum w dw) with equal dw: zero up to the rounding of the per-slot dw
    assert np.isfinite(dlog).all() and np.abs(dlog).max() < 1e-3


def test_gpt_oss_width_layer_matches_oracle(rp):
    """One layer at the full width of the GPT-OSS-20B-shaped workload (hidden = expert width = 2880, not a multiple of
    the 256-wide tiles; 64/8 heads of 64; 4 of 32 experts; router in the layer; LoRA r=8 on attention) on a short ragged
    sequence, against the oracle.  Decisive planted routing, as in the other router-in-the-layer tests."""
    B, H = rp
    c = synth.shrink(synth.CONFIGS["C6"], n_layers=1, seq=264)
    wl = synth.plant_routing(synth.make_workload(c, 1606, gains_random=True), c, 1606)
    ref = pu.oracle_chain(c, wl, dtype=np.float32)
    srt = -np.sort(-ref["logits"][0], axis=1)
    assert np.min(srt[:, c["top_k"] - 1] - srt[:, c["top_k"]]) > 0.05, "planted routing is not decisive"
    got = pu.gpu_chain(c, wl, H)
    errs = pu.compare_chain(ref, got, c)
    assert len(errs) == 2 + 2 + 2 * len(c["lora"]), sorted(errs)
