#!/usr/bin/env python3
"""Benchmark of the worker hot path on one MI355X: decoder-stage forward+backward (+ LM head with cross-entropy).

A step is one pass of the whole path over one micro-batch of a synthetic Qwen3-shaped stage: forward of the stage
keeping the internals, LM head + loss + its gradients (when the stage has a head), backward of the stage.  The default
workload is the largest one that fits one GPU, C4 (2 Qwen3-32B-shaped layers with LoRA r=16 on a frozen base + the
151936-entry LM head, 1 x 16384 tokens); its frozen weights are streamed from pinned host memory the way the paper's
worker receives them (Sec. 4.2): while a step computes on one device slot, the weights of the next stage call are being
uploaded into the other slot, in every timed step.  The activations (and the weights of the step itself) are resident
in HBM when the timed region starts.  The other workloads (C2 full fine-tune with resident weights, C3, C5) are measured
in the same run with fewer steps and reported as sub-records.

Prints ONE JSON line: tokens/s of the default workload, the roofline of its dominant kernel measured with HIP events
inside the library's per-kernel timeline, the CPU oracle timed on this machine's host cores on a bounded sample, and the
sub-records.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # 256 CUs x 4 SIMDs x 1024 FLOP/cycle x 2.4 GHz, dense
PEAK_HBM_GBS = 8000.0


def fl_gemm_fwd(c):
    """Projection FLOPs of one layer's forward (2*T*N*K each; MoE: every token runs top_k experts)."""
    T = c["batch"] * c["seq"]
    h, d, m = c["hidden"], c["head_dim"], c["ffn"]
    qd, kd = c["n_q_heads"] * d, c["n_kv_heads"] * d
    ffn_rows = T * c["top_k"] if c["n_experts"] else T
    router = 2.0 * T * c["n_experts"] * h if c.get("moe_router") else 0.0
    return 2.0 * T * (h * (qd + 2 * kd) + qd * h) + 2.0 * ffn_rows * (h * 2 * m + m * h) + router


def algorithmic_flops(c):
    """Useful FLOPs of one step.  Projections 2*T*N*K each, forward once and once more per gradient that is needed
    (activation gradient always, weight gradient with a trainable base; paper App. C.3); causal attention 2*s^2*qd
    forward per sequence and 2.5x that backward; LM head 4*T*h*V frozen (logits, dX), 6*T*h*V trainable (+ dW)."""
    T, s, b = c["batch"] * c["seq"], c["seq"], c["batch"]
    h, d, V = c["hidden"], c["head_dim"], c["vocab"]
    qd = c["n_q_heads"] * d
    attn_fwd = 2.0 * b * s * s * qd
    wgrad = 1.0 if c["train_base"] else 0.0
    layers = c["n_layers"] * (fl_gemm_fwd(c) * (2.0 + wgrad) + attn_fwd * 3.5)
    head = (4.0 + 2.0 * wgrad) * T * h * V if V else 0.0
    return layers, head


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc summary kept under profiles/ (FETCH_SIZE and WRITE_SIZE
    scaled by a copy kernel of known size), or None when that summary has no line for this workload and kernel.  A
    stored figure: counters cannot be read from inside this process."""
    path = os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic.md" % workload)
    try:
        with open(path) as f:
            for ln in f:
                w = ln.split()
                if len(w) >= 3 and w[0] == "traffic_bytes_per_launch" and w[1] == kernel:
                    return float(w[2])
    except OSError:
        pass
    return None


def cpu_baseline(c_full, sample_seq, seed):
    """The oracle as it stands (numpy fp32) on the same shapes with a shorter sequence; returns tokens/s and threads."""
    import numpy as np
    import synth
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import parity_util as pu
    c = synth.shrink(c_full, seq=sample_seq)
    wl = synth.make_workload(c, seed)
    threads = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        infos = [i for i in threadpool_info() if i.get("user_api") == "blas"]
        if infos:
            threads = infos[0]["num_threads"]
    except Exception:
        pass
    t0 = time.perf_counter()
    res = pu.oracle_chain(c, wl, dtype=np.float32)
    dt = time.perf_counter() - t0
    T = c["batch"] * c["seq"]
    note = "same stage%s (numpy fp32, forward+backward) at seq %d of %d, %d tokens in %.1f s" % (
        " and head" if c["vocab"] else "", sample_seq, c_full["seq"], T, dt)
    if "loss" in res:
        note += "; loss %.4f" % res["loss"]
    return {"value": T / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle", "sample": note}


def auto_cpu_seq(c):
    """Sequence length of the CPU sample: the longest power of two (at most the workload's) whose work is about 20 s at
    ~0.8 TFLOP/s of numpy fp32 on a 16-core host (10-30 s)."""
    import synth
    s = c["seq"]
    while s > 256:
        lay, head = algorithmic_flops(synth.shrink(c, seq=s))
        if (lay + head) / 0.8e12 <= 25.0:
            break
        s //= 2
    return s


def workload_text(name, c, has_head):
    return "%s: %d decoder layers (h=%d, %d/%d heads x %d, ffn %d%s)%s, batch %d x seq %d, %s" % (
        name, c["n_layers"], c["hidden"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"], c["ffn"],
        " x %d experts, top-%d%s" % (c["n_experts"], c["top_k"], ", router in the layer" if c.get("moe_router") else "") if c["n_experts"] else "",
        " + LM head V=%d with cross-entropy" % c["vocab"] if has_head else "", c["batch"], c["seq"],
        "full fine-tune, fp32 weight gradients" if c["train_base"] else "frozen base streamed from pinned host memory, LoRA r=%d" % c["lora_rank"])


def measure(name, args, steps, warmup, full):
    """One workload.  full: also the forward-stage, upload-sweep, multi-stream-round and CPU legs."""
    import numpy as np
    import torch
    import synth
    from paper_2604_27085_amd import binding as B
    from paper_2604_27085_amd import harness as H

    c = synth.CONFIGS[name]
    seed = synth.config_seed(name)

    def say(msg):          # progress on stderr: generating the larger workloads takes a while
        print("[bench %s] %s" % (name, msg), file=sys.stderr, flush=True)

    say("generating the synthetic workload on the host")
    wl = synth.make_workload(c, seed)
    has_head = wl["head"] is not None
    cfg = H.cfg_from_dict(c, with_head=has_head)
    R = H.StageRunner(cfg, c["batch"], c["seq"], n_slots=2)
    say("packing the weight blob (%.2f GB, pinned)" % (R.wbytes / 1e9))
    host = R.pinned_blob(wl["layers"], wl["head"])
    wl["layers"] = None
    wl["head"] = None
    x = H.bf16_tensor(wl["x"], R.device)
    dy_in = H.bf16_tensor(wl["dy"], R.device)
    labels = torch.from_numpy(wl["labels"]).to(R.device) if has_head else None
    router = None
    if wl.get("router_logits") is not None:
        router = torch.from_numpy(np.stack(wl["router_logits"])).to(R.device)
    elif c.get("moe_router"):      # the stage computes the logits into this buffer
        router = torch.empty((c["n_layers"], R.T, c["n_experts"]), dtype=torch.float32, device=R.device)
    d_router = torch.empty_like(router) if router is not None else None
    wl = None
    out = torch.empty_like(x)
    dx = torch.empty_like(x)
    dy_head = torch.empty_like(x)
    loss_buf = torch.empty(1, dtype=torch.float32, device=R.device)
    torch.cuda.synchronize()
    say("uploading %.2f GB of weights" % (R.wbytes / 1e9))
    t0 = time.perf_counter()
    R.upload(host, slot=0)
    R.copy.synchronize()
    t_up = time.perf_counter() - t0
    R.upload(host, slot=1)
    R.sync()
    T = R.T
    streamed = bool(c.get("stream"))

    def step(slot=0):
        if has_head:     # the fused last stage: recompute -> head on its own workspace -> backward (Sec. 3.2)
            return R.fused_last_stage(x, labels, out, dy_head, dx, loss_buf, 1.0, slot)
        B.rp_stage_backward(R.ctx, slot, B.PHASE_BOTH, x, dy_in, dx, out, R.grads if R.gbytes else None, router, d_router,
                            R.batch, R.seq, R.ws, R.wsbytes)
        return None

    def timed(n, with_upload):
        """n steps; with_upload: the upload for the next step streams into the other slot while each step computes."""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            if with_upload:
                R.upload(host, slot=(i + 1) & 1)
            loss = step(slot=i & 1 if with_upload else 0)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3, loss

    say("warm-up and timed steps%s" % (" (next upload in flight in every step)" if streamed else ""))
    for i in range(warmup):
        if streamed:
            R.upload(host, slot=(i + 1) & 1)
        step(slot=i & 1 if streamed else 0)
    if streamed and warmup & 1:      # leave the weights of the first timed step in slot 0
        R.upload(host, slot=0)
    ms_step, loss = timed(steps, streamed)
    loss_val = float(loss.item()) if loss is not None else None
    ms_resident = ms_step
    if streamed:
        R.upload(host, slot=0)
        ms_resident, _ = timed(max(2, min(steps, 5)), False)

    # ---- per-kernel timeline (HIP events recorded by the library on its compute stream), same steps, nothing else in flight
    tsteps = max(1, min(steps, 5))
    B.rp_trace_start(R.ctx, 4096 * tsteps)
    for _ in range(tsteps):
        step()
    recs = B.rp_trace_stop(R.ctx, 4096 * tsteps)
    agg = {}
    for kname, fl, by, ms in recs:
        a = agg.setdefault(kname, [0, 0.0, 0.0, 0.0])
        a[0] += 1
        a[1] += ms
        a[2] += fl
        a[3] += by
    traced_ms = sum(a[1] for a in agg.values()) / tsteps
    kernels = {}
    for kname, (n, ms, fl, by) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        kernels[kname] = {"calls_per_step": n / tsteps, "ms_per_step": round(ms / tsteps, 4), "avg_us": round(ms / n * 1e3, 2),
                          "tflops": round(fl / (ms * 1e-3) / 1e12, 1) if ms > 0 else 0.0,
                          "gbs": round(by / (ms * 1e-3) / 1e9, 1) if ms > 0 else 0.0}
    dname, (dn, dms, dfl, dby) = max(agg.items(), key=lambda kv: kv[1][1])
    if dfl > 0:
        ach = dfl / (dms * 1e-3) / 1e12
        roofline = {"kernel": dname, "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / PEAK_BF16_TFLOPS, 4)}
    else:
        ach = dby / (dms * 1e-3) / 1e9
        roofline = {"kernel": dname, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4)}
    roofline.update({"traffic": measured_traffic(name, dname),
                     "traffic_source": "stored figure: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, profiles/bench_%s_hbm_traffic.md" % name,
                     "launches_per_step": dn / tsteps, "avg_launch_us": round(dms / dn * 1e3, 2)})
    # class roll-ups against the targets: GEMMs and attention as fractions of the bf16 MFMA peak
    gemm_ms = sum(a[1] for k, a in agg.items() if k.startswith("gemm_"))
    gemm_fl = sum(a[2] for k, a in agg.items() if k.startswith("gemm_"))
    at_ms = sum(a[1] for k, a in agg.items() if k.startswith("attn_"))
    fl_layers, fl_head = algorithmic_flops(c)
    attn_alg = 7.0 * c["batch"] * c["seq"] ** 2 * c["n_q_heads"] * c["head_dim"] * c["n_layers"] * tsteps
    classes = {"gemm": {"ms_per_step": round(gemm_ms / tsteps, 3), "executed_tflops": round(gemm_fl / (gemm_ms * 1e-3) / 1e12, 1),
                        "frac_of_bf16_peak": round(gemm_fl / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}}
    if at_ms > 0:
        classes["attention"] = {"ms_per_step": round(at_ms / tsteps, 3), "algorithmic_tflops": round(attn_alg / (at_ms * 1e-3) / 1e12, 1),
                                "frac_of_bf16_peak": round(attn_alg / (at_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                "note": "all attention kernels (forward, delta, dQ, dK/dV and its reduce) against 7 s^2 qd FLOPs per layer"}
    mem = {k: v for k, v in kernels.items() if v["tflops"] == 0.0 and v["gbs"] > 0 and v["ms_per_step"] >= 0.02}
    classes["memory_bound"] = {k: {"gbs": v["gbs"], "frac_of_hbm_peak": round(v["gbs"] / PEAK_HBM_GBS, 3)} for k, v in mem.items()}

    tot_fl = fl_layers + fl_head
    rec = {
        "workload": workload_text(name, c, has_head), "tokens_per_step": T,
        "value": round(T / (ms_step * 1e-3), 1), "unit": "tokens/s", "steps": steps, "warmup": warmup, "ms_per_step": round(ms_step, 4),
        "upload_in_flight_in_timed_steps": streamed,
        "resident_ms_per_step": round(ms_resident, 4),
        "algorithmic_tflop_per_step": round(tot_fl / 1e12, 3), "tflops": round(tot_fl / (ms_step * 1e-3) / 1e12, 1),
        "frac_of_bf16_mfma_peak": round(tot_fl / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "loss": loss_val, "roofline": roofline, "classes": classes, "traced_ms_per_step": round(traced_ms, 3),
        "upload": {"bytes": R.wbytes, "h2d_gbs": round(R.wbytes / t_up / 1e9, 2), "upload_alone_ms": round(t_up * 1e3, 3),
                   "exposed_ms_at_one_micro_batch": round(max(0.0, ms_step - ms_resident), 3) if streamed else None,
                   "hidden_at_one_micro_batch": (ms_step - ms_resident <= 0.02 * ms_step) if streamed else None},
    }
    if full:
        rec["kernels"] = kernels
    else:
        rec["kernels"] = dict(list(kernels.items())[:8])

    # ---- forward stage alone (the F_i stages of Sec. 3.2: no internals kept, smaller workspace plan)
    if full and c["n_layers"] > 0 and not args.core_only:
        for _ in range(2):
            B.rp_stage_forward(R.ctx, 0, x, out, None, router, R.batch, R.seq, R.ws, R.wsbytes)
        torch.cuda.synchronize()
        nf = max(2, min(steps, 10))
        t0 = time.perf_counter()
        for _ in range(nf):
            B.rp_stage_forward(R.ctx, 0, x, out, None, router, R.batch, R.seq, R.ws, R.wsbytes)
        torch.cuda.synchronize()
        t_f = (time.perf_counter() - t0) / nf
        s_, qd_ = c["seq"], c["n_q_heads"] * c["head_dim"]
        fl_fwd = c["n_layers"] * (fl_gemm_fwd(c) + 2.0 * c["batch"] * s_ * s_ * qd_)
        rec["forward_stage"] = {"ms": round(t_f * 1e3, 3), "tokens_per_s": round(R.T / t_f, 1),
                                "algorithmic_tflops": round(fl_fwd / t_f / 1e12, 1)}

    # ---- weight streaming (Sec. 4.2): rounds of M_R micro-batches computed on one slot while the next stage's weights
    # stream into the other (Sec. 3.1: one upload serves M_R >= N micro-batches).  exposed = round time - M_R x the
    # resident-weights step; hidden when that is <= 2 % of the round.
    if full and not args.core_only:
        sweep, first_hidden = [], None
        for m_r in (1, 2, 4, 8):
            nrep = max(2, min(steps, 4 if m_r == 1 else 2))
            R.upload(host, slot=0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(nrep):
                R.upload(host, slot=(i + 1) & 1)     # next stage's weights stream in while this round computes
                for _ in range(m_r):
                    step(slot=i & 1)
            torch.cuda.synchronize()
            t_round = (time.perf_counter() - t0) / nrep * 1e3
            exposed = max(0.0, t_round - m_r * ms_resident)
            hidden = exposed <= 0.02 * t_round
            sweep.append({"m_r": m_r, "round_ms": round(t_round, 3), "exposed_ms": round(exposed, 3), "hidden": hidden})
            if hidden and first_hidden is None:
                first_hidden = m_r
            if hidden:
                break
        rec["upload"].update({"rounds": sweep, "smallest_m_r_hidden": first_hidden,
                              "note": "a round = one upload into the other slot while M_R micro-batches run on this one"})

    # ---- a round of the multi-stream worker (Sec. 4.2): backward stage over M_R micro-batches whose activations live in
    # pinned host memory, the next stage's weights streaming in and a finished gradient blob streaming out in the round's
    # windows.  Compared with the same M_R backward stages on device-resident activations and nothing else in flight.
    if full and not args.core_only and c["n_layers"] > 0 and not c["n_experts"]:
        m_r = args.round_micro
        R.enable_rounds(args.round_streams)
        pin = lambda: torch.empty((T, c["hidden"]), dtype=torch.bfloat16).pin_memory()
        xh, dyh, oh = [pin() for _ in range(m_r)], [pin() for _ in range(m_r)], [pin() for _ in range(m_r)]
        for t in xh:
            t.copy_(x)
        for t in dyh:
            t.copy_(dy_in)
        g_host = torch.empty(max(R.gbytes, 4) // 4, dtype=torch.float32).pin_memory() if R.gbytes else None
        g_done = torch.zeros_like(R.grads) if R.gbytes else None     # a finished stage's gradients, not the ones being accumulated

        def plain():
            for _ in range(m_r):
                B.rp_stage_backward(R.ctx, 0, B.PHASE_BOTH, x, dy_in, dx, out, R.grads if R.gbytes else None, None, None,
                                    R.batch, R.seq, R.ws, R.wsbytes)

        def rnd(i):
            R.round(xh, oh, slot=i & 1, dy_host=dyh, next_slot=(i + 1) & 1, next_host_blob=host,
                    done_grads_dev=g_done, done_grads_host=g_host,
                    max_piece_bytes=args.round_piece_mib << 20)

        R.upload(host, slot=0)
        plain()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plain()
        torch.cuda.synchronize()
        t_plain = (time.perf_counter() - t0) * 1e3
        rnd(0)
        R.sync()
        t0 = time.perf_counter()
        for i in range(1, 3):
            rnd(i)
        R.sync()
        t_round = (time.perf_counter() - t0) / 2 * 1e3
        moved = 3 * m_r * T * c["hidden"] * 2 + R.wbytes + R.gbytes
        rec["round"] = {"m_r": m_r, "round_ms": round(t_round, 3), "resident_ms": round(t_plain, 3),
                        "exposed_ms": round(max(0.0, t_round - t_plain), 3), "tokens_per_s": round(m_r * T / (t_round * 1e-3), 1),
                        "bytes_moved": moved, "link_gbs_if_serial": round(moved / (t_round * 1e-3) / 1e9, 1),
                        "note": "backward stage only (no head); per round: %d activation uploads (x, dy) and downloads (dx), the "
                                "whole weight blob up, the whole gradient blob down" % m_r}
        del xh, dyh, oh, g_host, g_done

    R.close()
    del R, host, x, dy_in, out, dx, dy_head, labels, router, d_router
    gc.collect()
    torch.cuda.empty_cache()

    if full and args.cpu_seq >= 0:
        cs = args.cpu_seq if args.cpu_seq > 0 else auto_cpu_seq(c)
        say("CPU oracle sample at seq %d" % cs)
        rec["cpu_baseline"] = cpu_baseline(c, min(cs, c["seq"]), seed)
    return rec


def gemm_probe(size, reps):
    """The projection GEMM alone at M = N = K = size, as NT and as NN: the four-wave kernel that loads its operands straight
    into LDS (tile 7, what the stage runs for long reductions), the staged eight-wave 256x256 kernel (tile 1) and the
    variant that streams a pre-arranged B operand past LDS (tile 6); for context the library product (torch.matmul) on
    the same box.  One JSON line; for counter runs (--gemm-reps 3)."""
    import torch
    from paper_2604_27085_amd import binding as B
    st = torch.cuda.current_stream().cuda_stream
    M = N = K = size
    a = (torch.randn(M, K, device="cuda") * 0.5).bfloat16()
    c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    out = {"probe": "gemm", "M": M, "N": N, "K": K, "reps": reps}

    def timed(fn):
        for _ in range(reps):     # untimed: the clock of a chip that was idle takes tens of milliseconds to settle
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        return {"us": round(us, 1), "tflops": round(2.0 * M * N * K / us / 1e6, 1)}

    for layout, lname in ((0, "NT"), (1, "NN")):
        b = (torch.randn((N, K) if layout == 0 else (K, N), device="cuda") * 0.05).bfloat16()
        ldb = K if layout == 0 else N
        arr = torch.empty(((N + 63) // 64) * ((K + 63) // 64) * 4096, dtype=torch.bfloat16, device="cuda")
        B.rp_op_gemm_arrange(st, b, ldb, N, K, layout, arr)
        variants = [(7, b, ldb, "lds_direct"), (1, b, ldb, "staged"), (6, arr, 0, "b_direct")]
        for tile, bb, l, tname in variants:
            out["%s_%s" % (lname, tname)] = timed(lambda: B.rp_op_gemm(st, layout, 0, a, bb, c, M, N, K, K, l, N, tile=tile))
        out["%s_library" % lname] = timed(lambda: torch.matmul(a, b.t() if layout == 0 else b, out=c))
    print(json.dumps(out))


def attn_probe(name, reps):
    """Attention alone at the shape of a workload (sequence, heads, head_dim 128): forward, then the backward (delta, dK/dV,
    its reduce, dQ) through the op-level entry points.  One JSON line; for counter runs (--attn-reps 2)."""
    import torch
    import synth
    from paper_2604_27085_amd import binding as B
    c = synth.CONFIGS[name]
    seq, a, kh, d, batch = c["seq"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"], c["batch"]
    T = batch * seq
    st = torch.cuda.current_stream().cuda_stream
    mk = lambda h: torch.randn(T, h * d, device="cuda").bfloat16()
    q, k, v, do = mk(a), mk(kh), mk(kh), mk(a)
    o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((batch, a, seq), dtype=torch.float32, device="cuda")
    delta = torch.empty_like(lse)
    scratch = torch.empty((2, T, a * d), dtype=torch.float32, device="cuda")
    fwd = lambda: B.rp_op_attn_fwd(st, q, k, v, o, lse, a * d, kh * d, kh * d, a * d, batch, seq, a, kh, d)
    bwd = lambda: B.rp_op_attn_bwd(st, q, k, v, o, do, lse, delta, dq, dk, dv, scratch, a * d, kh * d, kh * d, a * d, a * d,
                                   a * d, kh * d, kh * d, batch, seq, a, kh, d)
    unit = batch * float(seq) * seq * a * d          # FLOPs of one causal s x s x d product over all heads
    out = {"probe": "attention", "workload": name, "seq": seq, "heads": [a, kh], "head_dim": d, "reps": reps}
    for nm, fn, units in (("forward", fwd, 2.0), ("backward", bwd, 5.0)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        out[nm] = {"us": round(us, 1), "algorithmic_tflops": round(units * unit / us / 1e6, 1)}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C4", help="the workload of the headline figures")
    ap.add_argument("--others", default="C2,C3,C5", help="workloads reported as sub-records (comma separated; '' = none)")
    ap.add_argument("--cpu-seq", type=int, default=0, help="sequence length of the CPU-oracle sample (0 = about 20 s of work, -1 = skip)")
    ap.add_argument("--core-only", "--no-upload-leg", dest="core_only", action="store_true",
                    help="only the timed steps and the timeline steps of --config: no sub-records, no forward-stage, upload-sweep or round legs (profiling runs)")
    ap.add_argument("--round-streams", type=int, default=1, help="transfer streams per direction in the round leg (1 or 2)")
    ap.add_argument("--round-piece-mib", type=int, default=0, help="largest transfer piece in that leg (0 = the library's default)")
    ap.add_argument("--round-micro", type=int, default=4, help="micro-batches per round in the multi-stream leg")
    ap.add_argument("--gemm-probe", type=int, default=0, help="only time the square GEMM of this size, staged against B-direct, and exit")
    ap.add_argument("--gemm-reps", type=int, default=20)
    ap.add_argument("--attn-probe", default="", help="only time the attention kernels at this workload's shape (C2 .. C5) and exit")
    ap.add_argument("--attn-reps", type=int, default=5)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the one-GPU worker; a stage runs whole on one GPU and nothing here uses a "
              "second one, so --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.gemm_probe:
        gemm_probe(args.gemm_probe, args.gemm_reps)
        return
    if args.attn_probe:
        attn_probe(args.attn_probe, args.attn_reps)
        return

    main_rec = measure(args.config, args, args.steps, args.warmup, True)
    others = {}
    if not args.core_only:
        for name in [n for n in args.others.split(",") if n and n != args.config]:
            try:
                others[name] = measure(name, args, max(2, min(args.steps, 5)), max(1, min(args.warmup, 2)), False)
            except Exception as e:       # a sub-record must not cost the headline line
                others[name] = {"error": "%s: %s" % (type(e).__name__, e)}
    line = {
        "metric": "decoder-stage fwd+bwd tokens/s on 1 MI355X; MFMA % of bf16 peak",
        "value": main_rec["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": main_rec["workload"], "tokens_per_step": main_rec["tokens_per_step"],
                   "weights": "next stage call's weights uploading from pinned host memory during every timed step; this step's resident"
                   if main_rec["upload_in_flight_in_timed_steps"] else "resident in HBM"},
    }
    for k in ("resident_ms_per_step", "algorithmic_tflop_per_step", "tflops", "frac_of_bf16_mfma_peak", "loss", "roofline",
              "classes", "traced_ms_per_step", "kernels", "forward_stage", "upload", "round", "cpu_baseline"):
        if k in main_rec:
            line[k] = main_rec[k]
    line["other_workloads"] = others
    line["context"] = "paper reports only 8-GPU end-to-end speedups (1.48-2.16x on 8x RTX 4090); no per-stage number exists"
    print(json.dumps(line))


if __name__ == "__main__":
    main()
