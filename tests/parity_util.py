"""Shared helpers of the GPU parity tests: run one workload through the oracle and through the HIP library."""
import numpy as np

from oracle import StageConfig, stage


def oracle_cfg(c):
    return StageConfig(n_layers=c["n_layers"], hidden=c["hidden"], n_q_heads=c["n_q_heads"], n_kv_heads=c["n_kv_heads"],
                       head_dim=c["head_dim"], ffn=c["ffn"], vocab=c["vocab"], n_experts=c["n_experts"], top_k=c["top_k"],
                       rope_base=c.get("rope_base", 1.0e6), rms_eps=c.get("rms_eps", 1.0e-6), qk_norm=bool(c.get("qk_norm", 1)),
                       lora_rank=c["lora_rank"], lora_scale=c.get("lora_scale", 1.0), lora_targets=tuple(c["lora"]),
                       train_base=bool(c["train_base"]), moe_router=bool(c.get("moe_router", 0)))


def cast_tree(obj, dtype):
    if isinstance(obj, dict):
        return {k: cast_tree(v, dtype) for k, v in obj.items()}
    if isinstance(obj, (list, tuple)):
        return type(obj)(cast_tree(v, dtype) for v in obj)
    if isinstance(obj, np.ndarray) and obj.dtype.kind == "f":
        return obj.astype(dtype)
    return obj


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def oracle_chain(c, wl, dtype=np.float64, grad_scale=1.0):
    """stage forward -> (head loss, dx) -> stage backward; without a head, dy comes from the workload."""
    cfg = oracle_cfg(c)
    layers = cast_tree(wl["layers"], dtype)
    x = wl["x"].astype(dtype)
    router = None if wl.get("router_logits") is None else [r.astype(dtype) for r in wl["router_logits"]]
    res = {}
    if wl["head"] is not None:
        out, _ = stage.stage_fwd(x, layers, cfg, c["batch"], c["seq"], router)
        loss, dy, gh = stage.head_fwd_bwd(out, cast_tree(wl["head"], dtype), wl["labels"], cfg, grad_scale,
                                          want_dW=cfg.train_base)
        res.update(loss=float(loss), head_dx=dy, head_grads=gh)
    else:
        dy = wl["dy"].astype(dtype)
    if c["n_layers"] > 0:
        logits = []
        out, dx, grads = stage.stage_fwd_bwd(x, dy, layers, cfg, c["batch"], c["seq"], router, logits_out=logits)
        res.update(out=out, dx=dx, grads=grads)
        if cfg.moe_router:
            res["logits"] = logits
    return res


def gpu_chain(c, wl, harness, grad_scale=1.0, use_upload=True, fused=False):
    """fused: a stage with a head runs as the fused last stage (recompute -> head on its own workspace -> backward
    from the kept internals), the call sequence bench.py times, instead of forward stage -> head -> backward stage."""
    import torch
    cfg = harness.cfg_from_dict(c, with_head=wl["head"] is not None)
    R = harness.StageRunner(cfg, c["batch"], c["seq"])
    try:
        host = R.pinned_blob(wl["layers"], wl["head"])
        if use_upload:
            R.upload(host)
        else:
            R.slots[0].copy_(host)
            torch.cuda.synchronize()
            R.bind()
        x = harness.bf16_tensor(wl["x"], R.device)
        router = d_router = None
        if wl.get("router_logits") is not None:
            router = torch.from_numpy(np.stack(wl["router_logits"])).to(R.device)
            d_router = torch.full_like(router, float("nan"))
        elif c.get("moe_router"):     # the stage computes the logits into this buffer
            router = torch.full((c["n_layers"], R.T, c["n_experts"]), float("nan"), dtype=torch.float32, device=R.device)
            d_router = torch.full_like(router, float("nan"))
        torch.cuda.synchronize()
        res = {}
        if fused:
            assert wl["head"] is not None and c["n_layers"] > 0 and router is None
            labels = torch.from_numpy(wl["labels"]).to(R.device)
            out, dy, dx = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
            loss = torch.empty(1, dtype=torch.float32, device=R.device)
            torch.cuda.synchronize()
            R.fused_last_stage(x, labels, out, dy, dx, loss, grad_scale, train=bool(c["train_base"]))
            R.sync()
            res.update(loss=float(loss.item()), head_dx=harness.to_f32(dy), out=harness.to_f32(out), dx=harness.to_f32(dx))
            layer_g, head_g = harness.unpack_grads(cfg, R.grads)
            res.update(grads=layer_g, head_grads=head_g)
            return res
        if wl["head"] is not None:
            labels = torch.from_numpy(wl["labels"]).to(R.device)
            torch.cuda.synchronize()
            if c["n_layers"] > 0:
                out = R.forward(x, router=router)
            else:
                out = x
            loss, dy = R.head(out, labels, grad_scale, train=bool(c["train_base"]))
            R.sync()
            res.update(loss=float(loss.item()), head_dx=harness.to_f32(dy))
        else:
            dy = harness.bf16_tensor(wl["dy"], R.device)
            torch.cuda.synchronize()
        if c["n_layers"] > 0:
            out2, dx = R.backward(x, dy, router=router, d_router=d_router)
            R.sync()
            res.update(out=harness.to_f32(out2), dx=harness.to_f32(dx))
            if d_router is not None:
                res["d_router"] = d_router.cpu().numpy()
            if c.get("moe_router"):
                res["logits"] = router.cpu().numpy()
        R.sync()
        layer_g, head_g = harness.unpack_grads(cfg, R.grads)
        res.update(grads=layer_g, head_grads=head_g)
        return res
    finally:
        R.close()


def compare_chain(ref, got, c, tol=2e-2, loss_tol=1e-4, report=None):
    """Asserts the task's bounds: rel-L2 <= tol on outputs and every gradient tensor, |dloss|/|loss| <= loss_tol."""
    errs = {}
    if "loss" in ref:
        errs["loss"] = abs(got["loss"] - ref["loss"]) / abs(ref["loss"])
        errs["head_dx"] = rel_l2(got["head_dx"], ref["head_dx"])
        for k, v in ref["head_grads"].items():
            if k in got["head_grads"] and got["head_grads"][k] is not None:
                errs["head." + k] = rel_l2(got["head_grads"][k], v)
    if "out" in ref:
        errs["out"] = rel_l2(got["out"], ref["out"])
        errs["dx"] = rel_l2(got["dx"], ref["dx"])
        for li, lg in enumerate(ref.get("logits", [])):
            errs["L%d.logits" % li] = rel_l2(got["logits"][li], lg)
        for li, g in enumerate(ref["grads"]):
            gg = got["grads"][li]
            for k, v in g.items():
                if k == "router_logits":
                    errs["L%d.router_logits" % li] = rel_l2(got["d_router"][li], v)
                elif k == "lora":
                    for nm, (dA, dB) in v.items():
                        errs["L%d.lora.%s.A" % (li, nm)] = rel_l2(gg["lora"][nm][0], dA)
                        errs["L%d.lora.%s.B" % (li, nm)] = rel_l2(gg["lora"][nm][1], dB)
                elif k in gg and gg[k] is not None:
                    errs["L%d.%s" % (li, k)] = rel_l2(gg[k], v)
    if report is not None:
        report.update(errs)
    bad = {k: v for k, v in errs.items() if v > (loss_tol if k == "loss" else tol) or not np.isfinite(v)}
    assert not bad, "parity violations: %s\nall: %s" % (bad, errs)
    return errs
