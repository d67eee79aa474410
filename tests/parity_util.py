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


ROW_FACTOR, COLBLOCK_FACTOR, COLBLOCK = 4.0, 1.5, 256


def local_errors(got, ref):
    """Worst relative L2 error over single rows and over blocks of 256 columns of a tensor (1-D tensors: blocks of 256
    elements only).  A whole-tensor norm over thousands of rows cannot see one dead row or one wrong tail tile; these
    can.  Narrow tensors (LoRA factors [out, r], router-logit gradients with a few non-zeros per row) are taken in groups
    of rows that hold at least 256 elements, so that a norm has enough terms to mean something.  A row (block) is
    measured against the larger of its own reference norm and the root-mean-square norm of all rows (blocks): rows that
    are zero by construction (ignored labels) or small by cancellation carry rounding noise of the size of a typical
    row's, which is not an error of theirs."""
    a = np.asarray(got, dtype=np.float64)
    b = np.asarray(ref, dtype=np.float64)
    if a.ndim == 1:
        a, b = a[None, :], b[None, :]
    a = a.reshape(-1, a.shape[-1])
    b = b.reshape(-1, b.shape[-1])
    d = a - b
    out = {}
    if a.shape[0] > 1:
        grp = max(1, -(-COLBLOCK // a.shape[1]))        # rows per group
        ng = -(-a.shape[0] // grp)
        rs = lambda m: np.pad(np.einsum("ij,ij->i", m, m), (0, ng * grp - a.shape[0])).reshape(ng, grp).sum(axis=1)
        nr, er = np.sqrt(rs(b)), np.sqrt(rs(d))
        floor = np.sqrt(np.mean(nr * nr)) + 1e-30
        out["row"] = float(np.max(er / np.maximum(nr, floor)))
    nb = (a.shape[1] + COLBLOCK - 1) // COLBLOCK
    if nb > 1 or a.shape[0] == 1:
        pad = nb * COLBLOCK - a.shape[1]
        sq = lambda m: np.pad(np.einsum("ij,ij->j", m, m), (0, pad)).reshape(nb, COLBLOCK).sum(axis=1)
        nc, ec = np.sqrt(sq(b)), np.sqrt(sq(d))
        floor = np.sqrt(np.mean(nc * nc)) + 1e-30
        out["col"] = float(np.max(ec / np.maximum(nc, floor)))
    return out


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
            R.slots[0][:R.wbytes].copy_(host)
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


def chain_pairs(ref, got):
    """(name, got tensor, reference tensor) for every output and gradient of a chain result."""
    pairs = []
    if "loss" in ref:
        pairs.append(("head_dx", got["head_dx"], ref["head_dx"]))
        for k, v in ref["head_grads"].items():
            if k in got["head_grads"] and got["head_grads"][k] is not None:
                pairs.append(("head." + k, got["head_grads"][k], v))
    if "out" in ref:
        pairs.append(("out", got["out"], ref["out"]))
        pairs.append(("dx", got["dx"], ref["dx"]))
        for li, lg in enumerate(ref.get("logits", [])):
            pairs.append(("L%d.logits" % li, got["logits"][li], lg))
        for li, g in enumerate(ref["grads"]):
            gg = got["grads"][li]
            for k, v in g.items():
                if k == "router_logits":
                    pairs.append(("L%d.router_logits" % li, got["d_router"][li], v))
                elif k == "lora":
                    for nm, (dA, dB) in v.items():
                        pairs.append(("L%d.lora.%s.A" % (li, nm), gg["lora"][nm][0], dA))
                        pairs.append(("L%d.lora.%s.B" % (li, nm), gg["lora"][nm][1], dB))
                elif k in gg and gg[k] is not None:
                    pairs.append(("L%d.%s" % (li, k), gg[k], v))
    return pairs


def compare_chain(ref, got, c, tol=2e-2, loss_tol=1e-4, report=None, tol_of=None, local_report=None):
    """Asserts the task's bounds: rel-L2 <= tol on outputs and every gradient tensor, |dloss|/|loss| <= loss_tol; and
    beside every whole-tensor norm the local bounds of local_errors(): ROW_FACTOR * tol on every single row,
    COLBLOCK_FACTOR * tol on every block of 256 columns.  tol_of(name) may give a tensor its own bound."""
    errs, bad, loc = {}, {}, {}
    if "loss" in ref:
        errs["loss"] = abs(got["loss"] - ref["loss"]) / abs(ref["loss"])
        if not errs["loss"] <= loss_tol:
            bad["loss"] = errs["loss"]
    for name, g, r in chain_pairs(ref, got):
        t = tol_of(name) if tol_of is not None else tol
        errs[name] = rel_l2(g, r)
        if not errs[name] <= t:
            bad[name] = errs[name]
        for kind, v in local_errors(g, r).items():
            loc[name + "." + kind] = v / t
            if not v <= (ROW_FACTOR if kind == "row" else COLBLOCK_FACTOR) * t:
                bad[name + "." + kind] = v
    if report is not None:
        report.update(errs)
    if local_report is not None:
        local_report.update(loc)
    for kind in ("row", "col"):      # shown by pytest -s and on failure: how much room the local bounds leave
        w = max(((v, k) for k, v in loc.items() if k.endswith(kind)), default=None)
        if w:
            print("compare_chain: worst %s error %.2f x its tensor's bound (%s)" % (kind, w[0], w[1]))
    assert not bad, "parity violations: %s\nall: %s" % (bad, errs)
    return errs
