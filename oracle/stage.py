"""Stage-level oracle: a contiguous range of decoder layers, forward and backward with recomputation.

TEST INFRASTRUCTURE ONLY (see the package docstring).

A forward stage runs its layers on an incoming activation and hands on the boundary activation
(paper Sec. 3.2, asymmetric stage splitting).  A backward stage receives the stored stage input,
re-runs the forward keeping the internals, then back-propagates: recomputation, gradient w.r.t.
activations and gradient w.r.t. weights, each about one forward's worth of work (App. C.3).
Gradients accumulate in place across micro-batches (Sec. 4.1.1).

Per-layer parameters are a dict:
  g1, g2 [h]; Wq [qd,h]; Wk, Wv [kd,h]; Wo [h,qd]; gq, gk [d] (when cfg.qk_norm)
  dense:  Wg, Wu [m,h]; Wd [h,m]
  MoE:    Wg, Wu [E,m,h]; Wd [E,h,m]   (router logits are an input of the layer, or, with cfg.moe_router,
          logits = n2 Wr^T with the router Wr [E,h] a parameter of the layer: the "top-k softmax router" of the
          MoE layer in App. B.2 taken as one linear map of the normalised activation)
  lora:   {name: (A [r,in], B [out,r])} for name in cfg.lora_targets
"""
import numpy as np

from . import layers as L


def _lora(p, cfg, name):
    return p["lora"][name] if cfg.has_lora(name) else None


def layer_fwd(x, p, cfg, batch, seq, router_logits=None):
    """One decoder layer.  Returns the layer output and a cache of every internal needed by layer_bwd."""
    T = x.shape[0]
    a, kh, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    sc = cfg.lora_scale
    c = {"x": x}
    n1, c["rstd1"] = L.rmsnorm_fwd(x, p["g1"], cfg.rms_eps)
    c["n1"] = n1
    q = L.linear_fwd(n1, p["Wq"], _lora(p, cfg, "q"), sc).reshape(T, a, d)
    k = L.linear_fwd(n1, p["Wk"], _lora(p, cfg, "k"), sc).reshape(T, kh, d)
    v = L.linear_fwd(n1, p["Wv"], _lora(p, cfg, "v"), sc).reshape(T, kh, d)
    if cfg.qk_norm:
        c["q_raw"], c["k_raw"] = q, k
        q, c["rstd_q"] = L.rmsnorm_fwd(q, p["gq"], cfg.rms_eps)
        k, c["rstd_k"] = L.rmsnorm_fwd(k, p["gk"], cfg.rms_eps)
    q = L.rope_fwd(q, batch, seq, cfg.rope_base)
    k = L.rope_fwd(k, batch, seq, cfg.rope_base)
    o, P, lse = L.attention_fwd(q, k, v, batch, seq)
    c.update(q=q, k=k, v=v, o=o, P=P, lse=lse)
    o2 = o.reshape(T, a * d)
    y = x + L.linear_fwd(o2, p["Wo"], _lora(p, cfg, "o"), sc)
    c["y"] = y
    n2, c["rstd2"] = L.rmsnorm_fwd(y, p["g2"], cfg.rms_eps)
    c["n2"] = n2
    if cfg.n_experts > 0:
        if cfg.moe_router:
            router_logits = n2 @ p["Wr"].T
        c["logits"] = router_logits
        f, c["route"] = L.moe_ffn_fwd(n2, p["Wg"], p["Wu"], p["Wd"], router_logits, cfg.top_k)
        z = y + f
    else:
        gate = L.linear_fwd(n2, p["Wg"], _lora(p, cfg, "gate"), sc)
        up = L.linear_fwd(n2, p["Wu"], _lora(p, cfg, "up"), sc)
        act = L.swiglu_fwd(gate, up)
        c.update(gate=gate, up=up, act=act)
        z = y + L.linear_fwd(act, p["Wd"], _lora(p, cfg, "down"), sc)
    return z, c


def layer_bwd(dz, c, p, cfg, batch, seq):
    """Backward of layer_fwd.  Returns dx and a dict of gradients with the same keys as the parameters
    (base-weight gradients only when cfg.train_base; norm gains and LoRA factors always; for MoE also
    'router_logits')."""
    T = dz.shape[0]
    a, kh, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    sc = cfg.lora_scale
    tb = cfg.train_base
    g = {"lora": {}}

    def lin_bwd(dy, u, wname, lname):
        du, dW, dA, dB = L.linear_bwd(dy, u, p[wname], _lora(p, cfg, lname), sc, want_dW=tb)
        if tb:
            g[wname] = dW
        if cfg.has_lora(lname):
            g["lora"][lname] = (dA, dB)
        return du

    # z = y + FFN(n2)
    dy = dz.copy()
    if cfg.n_experts > 0:
        dn2, dlog, dWs = L.moe_ffn_bwd(dz, c["n2"], p["Wg"], p["Wu"], p["Wd"], c["route"], want_dW=tb)
        g["router_logits"] = dlog
        if cfg.moe_router:
            dn2 = dn2 + dlog @ p["Wr"]
            if tb:
                g["Wr"] = dlog.T @ c["n2"]
        if tb:
            g["Wg"], g["Wu"], g["Wd"] = dWs
    else:
        dact = lin_bwd(dz, c["act"], "Wd", "down")
        dgate, dup = L.swiglu_bwd(dact, c["gate"], c["up"])
        dn2 = lin_bwd(dgate, c["n2"], "Wg", "gate") + lin_bwd(dup, c["n2"], "Wu", "up")
    d_y, g["g2"] = L.rmsnorm_bwd(dn2, c["y"], p["g2"], c["rstd2"])
    dy += d_y
    # y = x + Lin_o(o)
    dx = dy.copy()
    do = lin_bwd(dy, c["o"].reshape(T, a * d), "Wo", "o").reshape(T, a, d)
    dq, dk, dv = L.attention_bwd(do, c["q"], c["k"], c["v"], c["o"], c["P"], batch, seq)
    dq = L.rope_bwd(dq, batch, seq, cfg.rope_base)
    dk = L.rope_bwd(dk, batch, seq, cfg.rope_base)
    if cfg.qk_norm:
        dq, g["gq"] = L.rmsnorm_bwd(dq, c["q_raw"], p["gq"], c["rstd_q"])
        dk, g["gk"] = L.rmsnorm_bwd(dk, c["k_raw"], p["gk"], c["rstd_k"])
    dn1 = lin_bwd(dq.reshape(T, a * d), c["n1"], "Wq", "q")
    dn1 = dn1 + lin_bwd(dk.reshape(T, kh * d), c["n1"], "Wk", "k")
    dn1 = dn1 + lin_bwd(dv.reshape(T, kh * d), c["n1"], "Wv", "v")
    d_x, g["g1"] = L.rmsnorm_bwd(dn1, c["x"], p["g1"], c["rstd1"])
    dx += d_x
    return dx, g


def stage_fwd(x, params, cfg, batch, seq, router_logits=None, logits_out=None):
    """Forward of layers params[0..L-1].  Returns the boundary activation and the list of each layer's input.
    logits_out: optional list that receives every MoE layer's router logits."""
    layer_inputs = []
    for li, p in enumerate(params):
        layer_inputs.append(x)
        rl = None if router_logits is None else router_logits[li]
        x, c = layer_fwd(x, p, cfg, batch, seq, rl)
        if logits_out is not None:
            logits_out.append(c.get("logits"))
    return x, layer_inputs


def stage_fwd_bwd(x_in, dy, params, cfg, batch, seq, router_logits=None, logits_out=None):
    """Backward stage with recomputation: forward keeping internals, then backward in reverse order.
    Returns the stage output, dx and the per-layer gradient dicts."""
    caches = []
    x = x_in
    for li, p in enumerate(params):
        rl = None if router_logits is None else router_logits[li]
        x, c = layer_fwd(x, p, cfg, batch, seq, rl)
        if logits_out is not None:
            logits_out.append(c.get("logits"))
        caches.append(c)
    out = x
    grads = [None] * len(params)
    d = dy
    for li in reversed(range(len(params))):
        d, grads[li] = layer_bwd(d, caches[li], params[li], cfg, batch, seq)
        caches[li] = None
    return out, d, grads


def head_fwd_bwd(x, head, labels, cfg, grad_scale=1.0, want_dW=True):
    """LM head (+ optional final norm gain head['gf']) fused with the mean cross-entropy.
    Returns loss, dx, dict of gradients {'Wv', 'gf'}."""
    loss, dx, dWv, dgf = L.lmhead_ce_fwd_bwd(x, head["Wv"], labels, head.get("gf"), cfg.rms_eps,
                                             grad_scale, want_dW)
    g = {}
    if want_dW:
        g["Wv"] = dWv
    if dgf is not None:
        g["gf"] = dgf
    return loss, dx, g
