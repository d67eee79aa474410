#!/usr/bin/env python3
"""Benchmark of the worker hot path on one MI355X: decoder-stage forward+backward plus LM head with cross-entropy.

A step is one pass of the whole path over one micro-batch of the Qwen3-1.7B-shaped workload (4 decoder layers,
hidden 2048, 16/8 heads of 128, FFN 6144, vocabulary 151936, batch 1 x 4096 tokens, full fine-tune in bf16 with fp32
weight gradients): forward of the stage keeping the internals, LM head + loss + its gradients, backward of the stage.
Weights are resident in HBM when the timed region starts (they were put there by rp_stage_upload_weights).

Prints ONE JSON line: tokens/s, the roofline of the dominant kernel measured with HIP events inside the library's
per-kernel timeline, and the CPU oracle timed on this machine's host cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # 256 CUs x 4 SIMDs x 1024 FLOP/cycle x 2.4 GHz, dense
PEAK_HBM_GBS = 8000.0


def algorithmic_flops(c):
    """Useful FLOPs of one step.  Projections 2*T*N*K each, forward once and twice more for the two gradients (paper
    App. C.3); causal attention 2*s^2*qd forward per sequence and 2.5x that backward; LM head 6*T*h*V (logits once, dX, dW)."""
    T, s, b = c["batch"] * c["seq"], c["seq"], c["batch"]
    h, d, m, V = c["hidden"], c["head_dim"], c["ffn"], c["vocab"]
    qd, kd = c["n_q_heads"] * d, c["n_kv_heads"] * d
    gemm_fwd = fl_gemm_fwd(c)
    attn_fwd = 2.0 * b * s * s * qd
    wgrad = 1.0 if c["train_base"] else 0.0
    layers = c["n_layers"] * (gemm_fwd * (2.0 + wgrad) + attn_fwd * 3.5)
    head = (4.0 + 2.0 * wgrad) * T * h * V if V else 0.0
    return layers, head


def fl_gemm_fwd(c):
    """Projection FLOPs of one layer's forward (2*T*N*K each; MoE: every token runs top_k experts)."""
    T = c["batch"] * c["seq"]
    h, d, m = c["hidden"], c["head_dim"], c["ffn"]
    qd, kd = c["n_q_heads"] * d, c["n_kv_heads"] * d
    ffn_rows = T * c["top_k"] if c["n_experts"] else T
    router = 2.0 * T * c["n_experts"] * h if c.get("moe_router") else 0.0
    return 2.0 * T * (h * (qd + 2 * kd) + qd * h) + 2.0 * ffn_rows * (h * 2 * m + m * h) + router


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc summary kept under profiles/ (FETCH_SIZE and WRITE_SIZE
    scaled by a copy kernel of known size), or None when that summary has no line for this workload and kernel."""
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
    return {"value": T / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "same stage and head (numpy fp32, forward+backward) at seq %d of %d, %d tokens in %.1f s; loss %.4f"
                      % (sample_seq, c_full["seq"], T, dt, res["loss"])}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--cpu-seq", type=int, default=4096, help="sequence length of the CPU-oracle sample (0 = skip)")
    ap.add_argument("--no-upload-leg", "--core-only", dest="no_upload_leg", action="store_true",
                    help="only the timed steps and the timeline steps: no forward-stage, upload or round legs (profiling runs)")
    ap.add_argument("--round-streams", type=int, default=1, help="transfer streams per direction in that leg (1 or 2)")
    ap.add_argument("--round-piece-mib", type=int, default=0, help="largest transfer piece in that leg (0 = the library's default)")
    ap.add_argument("--round-micro", type=int, default=4, help="micro-batches per round in the multi-stream leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the one-GPU worker; a stage runs whole on one GPU and nothing here uses a "
              "second one, so --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from paper_2604_27085_amd import binding as B
    from paper_2604_27085_amd import harness as H

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    c = synth.CONFIGS[args.config]
    seed = synth.config_seed(args.config)

    def say(msg):          # progress on stderr: generating the larger workloads takes a while
        print("[bench %s] %s" % (args.config, msg), file=sys.stderr, flush=True)

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
    out = torch.empty_like(x)
    dx = torch.empty_like(x)
    dy_head = torch.empty_like(x)
    loss_buf = torch.empty(1, dtype=torch.float32, device=R.device)
    torch.cuda.synchronize()
    say("uploading %.2f GB of weights" % (R.wbytes / 1e9))
    R.upload(host, slot=0)
    R.sync()
    T = R.T
    losses = []

    def step(slot=0):
        if has_head:
            return R.fused_last_stage(x, labels, out, dy_head, dx, loss_buf, 1.0, slot)
        B.rp_stage_backward(R.ctx, slot, B.PHASE_BOTH, x, dy_in, dx, out, R.grads if R.gbytes else None, router, d_router,
                            R.batch, R.seq, R.ws, R.wsbytes)
        return None

    say("warm-up and timed steps")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / args.steps * 1e3
    loss_val = float(loss.item()) if loss is not None else None

    # ---- per-kernel timeline (HIP events recorded by the library on its compute stream), same steps again
    tsteps = max(1, min(args.steps, 5))
    B.rp_trace_start(R.ctx, 4096 * tsteps)
    for _ in range(tsteps):
        step()
    recs = B.rp_trace_stop(R.ctx, 4096 * tsteps)
    agg = {}
    for name, fl, by, ms in recs:
        a = agg.setdefault(name, [0, 0.0, 0.0, 0.0])
        a[0] += 1
        a[1] += ms
        a[2] += fl
        a[3] += by
    traced_ms = sum(a[1] for a in agg.values()) / tsteps
    kernels = {}
    for name, (n, ms, fl, by) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        kernels[name] = {"calls_per_step": n / tsteps, "ms_per_step": round(ms / tsteps, 4), "avg_us": round(ms / n * 1e3, 2),
                         "tflops": round(fl / (ms * 1e-3) / 1e12, 1) if ms > 0 else 0.0,
                         "gbs": round(by / (ms * 1e-3) / 1e9, 1) if ms > 0 else 0.0}
    dom = max(agg.items(), key=lambda kv: kv[1][1])
    dname, (dn, dms, dfl, dby) = dom
    if dfl > 0:
        ach = dfl / (dms * 1e-3) / 1e12
        roofline = {"kernel": dname, "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": None, "launches_per_step": dn / tsteps,
                    "avg_launch_us": round(dms / dn * 1e3, 2)}
    else:
        ach = dby / (dms * 1e-3) / 1e9
        roofline = {"kernel": dname, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None, "launches_per_step": dn / tsteps,
                    "avg_launch_us": round(dms / dn * 1e3, 2)}
    roofline["traffic"] = measured_traffic(args.config, dname)
    # class roll-ups against the targets: GEMMs and attention as fractions of the bf16 MFMA peak
    gemm_ms = sum(a[1] for k, a in agg.items() if k.startswith("gemm_"))
    gemm_fl = sum(a[2] for k, a in agg.items() if k.startswith("gemm_"))
    at_ms = sum(a[1] for k, a in agg.items() if k.startswith("attn_fwd") or k.startswith("attn_bwd"))
    fl_layers, fl_head = algorithmic_flops(c)
    attn_alg = 7.0 * c["batch"] * c["seq"] ** 2 * c["n_q_heads"] * c["head_dim"] * c["n_layers"] * tsteps
    classes = {
        "gemm": {"ms_per_step": round(gemm_ms / tsteps, 3), "executed_tflops": round(gemm_fl / (gemm_ms * 1e-3) / 1e12, 1),
                 "frac_of_bf16_peak": round(gemm_fl / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
        "attention": {"ms_per_step": round(at_ms / tsteps, 3), "algorithmic_tflops": round(attn_alg / (at_ms * 1e-3) / 1e12, 1),
                      "frac_of_bf16_peak": round(attn_alg / (at_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
    }

    # ---- forward stage alone (the F_i stages of Sec. 3.2: no internals kept, smaller workspace plan)
    fwd_stage = None
    if c["n_layers"] > 0 and not args.no_upload_leg:
        for _ in range(2):
            B.rp_stage_forward(R.ctx, 0, x, out, None, router, R.batch, R.seq, R.ws, R.wsbytes)
        torch.cuda.synchronize()
        nf = max(2, min(args.steps, 10))
        t0 = time.perf_counter()
        for _ in range(nf):
            B.rp_stage_forward(R.ctx, 0, x, out, None, router, R.batch, R.seq, R.ws, R.wsbytes)
        torch.cuda.synchronize()
        t_f = (time.perf_counter() - t0) / nf
        s_, qd_ = c["seq"], c["n_q_heads"] * c["head_dim"]
        fl_fwd = c["n_layers"] * (fl_gemm_fwd(c) + 2.0 * c["batch"] * s_ * s_ * qd_)
        fwd_stage = {"ms": round(t_f * 1e3, 3), "tokens_per_s": round(R.T / t_f, 1),
                     "algorithmic_tflops": round(fl_fwd / t_f / 1e12, 1)}

    # ---- weight streaming (Sec. 4.2): H2D rate of rp_stage_upload_weights alone, then rounds of M_R micro-batches
    # computed on one slot while the next stage's weights stream into the other (Sec. 3.1: one upload serves M_R >= N
    # micro-batches).  exposed = round time - M_R x the resident-weights step; hidden when that is <= 2 % of the round.
    upload = None
    if not args.no_upload_leg:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        R.upload(host, slot=1)
        R.copy.synchronize()
        t_up = time.perf_counter() - t0
        sweep, first_hidden = [], None
        for m_r in (1, 2, 4, 8):
            nrep = max(2, min(args.steps, 6 if m_r == 1 else 3))
            R.upload(host, slot=0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(nrep):
                R.upload(host, slot=(i + 1) & 1)     # next stage's weights stream in while this round computes
                for _ in range(m_r):
                    step(slot=i & 1)
            torch.cuda.synchronize()
            t_round = (time.perf_counter() - t0) / nrep * 1e3
            exposed = max(0.0, t_round - m_r * ms_step)
            hidden = exposed <= 0.02 * t_round
            sweep.append({"m_r": m_r, "round_ms": round(t_round, 3), "exposed_ms": round(exposed, 3), "hidden": hidden})
            if hidden and first_hidden is None:
                first_hidden = m_r
            if hidden and m_r >= 2:
                break
        upload = {"bytes": R.wbytes, "h2d_gbs": round(R.wbytes / t_up / 1e9, 2), "upload_alone_ms": round(t_up * 1e3, 3),
                  "step_with_upload_in_flight_ms": sweep[0]["round_ms"], "exposed_ms": sweep[0]["exposed_ms"],
                  "rounds": sweep, "smallest_m_r_hidden": first_hidden,
                  "note": "a round = one upload into the other slot while M_R micro-batches run on this one"}

    # ---- a round of the multi-stream worker (Sec. 4.2): backward stage over M_R micro-batches whose activations live in
    # pinned host memory, the next stage's weights streaming in and a finished gradient blob streaming out in the round's
    # windows.  Compared with the same M_R backward stages on device-resident activations and nothing else in flight.
    round_leg = None
    if not args.no_upload_leg and c["n_layers"] > 0 and not c["n_experts"]:
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
        for _ in range(2):
            plain()
        torch.cuda.synchronize()
        t_plain = (time.perf_counter() - t0) / 2 * 1e3
        rnd(0)
        R.sync()
        t0 = time.perf_counter()
        for i in range(1, 4):
            rnd(i)
        R.sync()
        t_round = (time.perf_counter() - t0) / 3 * 1e3
        moved = 3 * m_r * T * c["hidden"] * 2 + R.wbytes + R.gbytes
        round_leg = {"m_r": m_r, "round_ms": round(t_round, 3), "resident_ms": round(t_plain, 3),
                     "exposed_ms": round(max(0.0, t_round - t_plain), 3), "tokens_per_s": round(m_r * T / (t_round * 1e-3), 1),
                     "bytes_moved": moved, "link_gbs_if_serial": round(moved / (t_round * 1e-3) / 1e9, 1),
                     "note": "backward stage only (no head); per round: %d activation uploads (x, dy) and downloads (dx), the "
                             "whole weight blob up, the whole gradient blob down" % m_r}

    cpu = None
    if args.cpu_seq > 0:
        say("CPU oracle sample")
        cpu = cpu_baseline(c, min(args.cpu_seq, c["seq"]), seed)

    tot_fl = fl_layers + fl_head
    line = {
        "metric": "decoder-stage fwd+bwd tokens/s on 1 MI355X; MFMA % of bf16 peak",
        "value": round(T / (ms_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: %d decoder layers (h=%d, %d/%d heads x %d, ffn %d%s)%s, batch %d x seq %d, "
                               "%s" % (args.config, c["n_layers"], c["hidden"], c["n_q_heads"], c["n_kv_heads"],
                                       c["head_dim"], c["ffn"],
                                       " x %d experts, top-%d%s" % (c["n_experts"], c["top_k"], ", router in the layer" if c.get("moe_router") else "") if c["n_experts"] else "",
                                       " + LM head V=%d with cross-entropy" % c["vocab"] if has_head else "",
                                       c["batch"], c["seq"],
                                       "full fine-tune, fp32 weight gradients" if c["train_base"] else "frozen base, LoRA r=%d" % c["lora_rank"]),
                   "tokens_per_step": T, "weights_resident_in_hbm": True},
        "algorithmic_tflop_per_step": round(tot_fl / 1e12, 3),
        "tflops": round(tot_fl / (ms_step * 1e-3) / 1e12, 1),
        "frac_of_bf16_mfma_peak": round(tot_fl / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "loss": loss_val,
        "roofline": roofline, "classes": classes, "traced_ms_per_step": round(traced_ms, 3), "kernels": kernels,
        "forward_stage": fwd_stage, "upload": upload, "round": round_leg, "cpu_baseline": cpu,
        "context": "paper reports only 8-GPU end-to-end speedups (1.48-2.16x on 8x RTX 4090); no per-stage number exists",
    }
    R.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
