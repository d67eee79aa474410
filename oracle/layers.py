"""Layer-level definitions of the oracle, forward and hand-derived backward (numpy).

TEST INFRASTRUCTURE ONLY (see the package docstring).  The paper treats a transformer layer as a
unit of work whose forward consists of the Q/K/V/output projections, attention and the three FFN
projections (App. B.2, Eq. flops-dense) and whose backward is "recompute + gradient w.r.t.
activations + gradient w.r.t. weights" (App. C.3).  The element-level definitions below are the
public Qwen3-style ones.  The working dtype is that of the arrays passed in (fp64 in tests, fp32
when timed); nothing is blocked, fused or re-ordered.

Conventions: x is [T, features] with T = batch*seq (sequence-major inside a batch entry);
weights are [out, in]; LoRA A is [r, in], B is [out, r]; heads are laid out [T, heads, d].
"""
import numpy as np


# ----------------------------------------------------------------------------- RMSNorm
def rmsnorm_fwd(x, g, eps):
    """y = x * rstd * g with rstd_t = (mean_j x_tj^2 + eps)^(-1/2), over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(ms + eps)
    return x * rstd * g, rstd


def rmsnorm_bwd(dy, x, g, rstd):
    """dx = rstd*(dy*g) - rstd^3/n * x * sum_j(dy_j g_j x_j);  dg = sum over rows of dy * x * rstd."""
    n = x.shape[-1]
    dyg = dy * g
    dot = np.sum(dyg * x, axis=-1, keepdims=True)
    dx = rstd * dyg - (rstd ** 3) * x * dot / n
    dg = np.sum((dy * x * rstd).reshape(-1, n), axis=0)
    return dx, dg


# ----------------------------------------------------------------------------- Linear (+LoRA)
def linear_fwd(u, W, lora=None, scale=1.0):
    """y = u W^T (+ scale * (u A^T) B^T when lora=(A, B))."""
    y = u @ W.T
    if lora is not None:
        A, B = lora
        y = y + scale * ((u @ A.T) @ B.T)
    return y


def linear_bwd(dy, u, W, lora=None, scale=1.0, want_dW=True):
    """Returns du, dW (or None), dA, dB (None without LoRA)."""
    du = dy @ W
    dW = dy.T @ u if want_dW else None
    dA = dB = None
    if lora is not None:
        A, B = lora
        dyB = dy @ B                      # [T, r]
        du = du + scale * (dyB @ A)
        dB = scale * (dy.T @ (u @ A.T))   # [out, r]
        dA = scale * (dyB.T @ u)          # [r, in]
    return du, dW, dA, dB


# ----------------------------------------------------------------------------- RoPE
def rope_angles(seq, d, base, dtype):
    """phi[p, i] = p * base^(-2i/d), p = 0..seq-1, i = 0..d/2-1 (half-split pairing (i, i+d/2))."""
    i = np.arange(d // 2, dtype=np.float64)
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * i / d)
    p = np.arange(seq, dtype=np.float64)[:, None]
    phi = p * theta[None, :]
    return np.cos(phi).astype(dtype), np.sin(phi).astype(dtype)


def rope_fwd(u, batch, seq, base):
    """u: [T, H, d].  Rotates pair (u_i, u_{i+d/2}) by angle pos*theta_i; positions restart per sequence."""
    T, H, d = u.shape
    cos, sin = rope_angles(seq, d, base, u.dtype)
    u = u.reshape(batch, seq, H, d)
    a, b = u[..., : d // 2], u[..., d // 2:]
    c = cos[None, :, None, :]
    s = sin[None, :, None, :]
    out = np.concatenate([a * c - b * s, b * c + a * s], axis=-1)
    return out.reshape(T, H, d)


def rope_bwd(dout, batch, seq, base):
    """Transpose of the rotation = rotation by the negative angle."""
    T, H, d = dout.shape
    cos, sin = rope_angles(seq, d, base, dout.dtype)
    g = dout.reshape(batch, seq, H, d)
    ga, gb = g[..., : d // 2], g[..., d // 2:]
    c = cos[None, :, None, :]
    s = sin[None, :, None, :]
    du = np.concatenate([ga * c + gb * s, gb * c - ga * s], axis=-1)
    return du.reshape(T, H, d)


# ----------------------------------------------------------------------------- causal GQA attention
def attention_fwd(q, k, v, batch, seq):
    """q: [T, a, d]; k, v: [T, kh, d].  Query head j uses kv head j // (a/kh).
    S = q k^T / sqrt(d), masked to t' <= t inside each sequence, P = softmax rows, o = P v.
    Returns o [T, a, d], the list of P matrices (per batch entry, per head) and LSE [batch, a, seq]."""
    T, a, d = q.shape
    kh = k.shape[1]
    grp = a // kh
    o = np.empty_like(q)
    lse = np.empty((batch, a, seq), dtype=q.dtype)
    P_all = []
    mask = np.triu(np.ones((seq, seq), dtype=bool), k=1)
    inv = 1.0 / np.sqrt(np.asarray(d, dtype=q.dtype))
    for bi in range(batch):
        sl = slice(bi * seq, (bi + 1) * seq)
        row = []
        for j in range(a):
            S = (q[sl, j, :] @ k[sl, j // grp, :].T) * inv
            S = np.where(mask, -np.inf, S)
            m = np.max(S, axis=-1, keepdims=True)
            e = np.exp(S - m)
            l = np.sum(e, axis=-1, keepdims=True)
            P = e / l
            o[sl, j, :] = P @ v[sl, j // grp, :]
            lse[bi, j, :] = (m + np.log(l))[:, 0]
            row.append(P)
        P_all.append(row)
    return o, P_all, lse


def attention_bwd(do, q, k, v, o, P_all, batch, seq):
    """dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(dO*O)), dQ = dS K / sqrt(d), dK = dS^T Q / sqrt(d);
    dK and dV are summed over the query heads that share a kv head."""
    T, a, d = q.shape
    kh = k.shape[1]
    grp = a // kh
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    inv = 1.0 / np.sqrt(np.asarray(d, dtype=q.dtype))
    for bi in range(batch):
        sl = slice(bi * seq, (bi + 1) * seq)
        for j in range(a):
            g = j // grp
            P = P_all[bi][j]
            dO = do[sl, j, :]
            dv[sl, g, :] += P.T @ dO
            dP = dO @ v[sl, g, :].T
            D = np.sum(dO * o[sl, j, :], axis=-1, keepdims=True)
            dS = P * (dP - D)
            dq[sl, j, :] = (dS @ k[sl, g, :]) * inv
            dk[sl, g, :] += (dS.T @ q[sl, j, :]) * inv
    return dq, dk, dv


# ----------------------------------------------------------------------------- SwiGLU
def sigmoid(t):
    return 1.0 / (1.0 + np.exp(-t))


def swiglu_fwd(gate, up):
    """act = silu(gate) * up, silu(t) = t / (1 + e^-t)."""
    return gate * sigmoid(gate) * up


def swiglu_bwd(dact, gate, up):
    sg = sigmoid(gate)
    dgate = dact * up * sg * (1.0 + gate * (1.0 - sg))
    dup = dact * gate * sg
    return dgate, dup


# ----------------------------------------------------------------------------- top-k MoE FFN
def moe_route(logits, top_k):
    """Indices of the top_k largest logits per row (ties -> lower expert index first) and the
    softmax over just those logits.  Returns idx [T, top_k] (descending logit), w [T, top_k]."""
    T, E = logits.shape
    order = np.argsort(-logits, axis=-1, kind="stable")[:, :top_k]
    sel = np.take_along_axis(logits, order, axis=-1)
    sel = sel - np.max(sel, axis=-1, keepdims=True)
    e = np.exp(sel)
    w = e / np.sum(e, axis=-1, keepdims=True)
    return order, w


def moe_ffn_fwd(n2, Wg, Wu, Wd, logits, top_k):
    """out_t = sum_{e in I_t} w_te * Wd_e (silu(Wg_e n2_t) * (Wu_e n2_t)).  Wg, Wu: [E, m, h]; Wd: [E, h, m]."""
    T, h = n2.shape
    idx, w = moe_route(logits, top_k)
    out = np.zeros_like(n2)
    cache = []
    for t in range(T):
        per = []
        for j in range(top_k):
            e = idx[t, j]
            gt = Wg[e] @ n2[t]
            ut = Wu[e] @ n2[t]
            at = gt * sigmoid(gt) * ut
            ft = Wd[e] @ at
            out[t] += w[t, j] * ft
            per.append((e, gt, ut, at, ft))
        cache.append(per)
    return out, (idx, w, cache)


def moe_ffn_bwd(dout, n2, Wg, Wu, Wd, route_cache, want_dW=False):
    """Returns dn2, dlogits [T, E] and (dWg, dWu, dWd) when want_dW.
    dw_te = <dout_t, FFN_e(n2_t)>;  dlogit_te = w_te (dw_te - sum_e' w_te' dw_te') on selected experts, else 0."""
    idx, w, cache = route_cache
    T, h = n2.shape
    E = Wg.shape[0]
    top_k = idx.shape[1]
    dn2 = np.zeros_like(n2)
    dlogits = np.zeros((T, E), dtype=n2.dtype)
    dWg = np.zeros_like(Wg) if want_dW else None
    dWu = np.zeros_like(Wu) if want_dW else None
    dWd = np.zeros_like(Wd) if want_dW else None
    for t in range(T):
        dw = np.zeros(top_k, dtype=n2.dtype)
        for j in range(top_k):
            e, gt, ut, at, ft = cache[t][j]
            dw[j] = np.dot(dout[t], ft)
            dft = w[t, j] * dout[t]
            dat = Wd[e].T @ dft
            sg = sigmoid(gt)
            dgt = dat * ut * sg * (1.0 + gt * (1.0 - sg))
            dut = dat * gt * sg
            dn2[t] += Wg[e].T @ dgt + Wu[e].T @ dut
            if want_dW:
                dWd[e] += np.outer(dft, at)
                dWg[e] += np.outer(dgt, n2[t])
                dWu[e] += np.outer(dut, n2[t])
        mix = np.dot(w[t], dw)
        for j in range(top_k):
            dlogits[t, idx[t, j]] = w[t, j] * (dw[j] - mix)
    return dn2, dlogits, (dWg, dWu, dWd)


# ----------------------------------------------------------------------------- LM head + cross-entropy
IGNORE_INDEX = -100


def lmhead_ce_fwd_bwd(x, Wv, labels, gf=None, eps=1e-6, grad_scale=1.0, want_dW=True):
    """xf = rmsnorm(x; gf) if gf is given; Z = xf Wv^T; loss = mean over valid rows of (logsumexp(Z_t) - Z[t, y_t]);
    dZ = grad_scale * (softmax(Z) - onehot) / N_valid on valid rows, 0 on rows labelled IGNORE_INDEX.
    Returns loss, dx, dWv (or None), dgf (or None)."""
    if gf is not None:
        xf, rstd = rmsnorm_fwd(x, gf, eps)
    else:
        xf = x
    Z = xf @ Wv.T
    valid = labels != IGNORE_INDEX
    n_valid = int(np.sum(valid))
    m = np.max(Z, axis=-1, keepdims=True)
    e = np.exp(Z - m)
    ssum = np.sum(e, axis=-1, keepdims=True)
    lse = (m + np.log(ssum))[:, 0]
    rows = np.nonzero(valid)[0]
    picked = Z[rows, labels[rows]]
    loss = np.sum(lse[rows] - picked) / max(n_valid, 1)
    dZ = e / ssum
    dZ[rows, labels[rows]] -= 1.0
    dZ[~valid, :] = 0.0
    dZ *= grad_scale / max(n_valid, 1)
    dxf = dZ @ Wv
    dWv = dZ.T @ xf if want_dW else None
    if gf is not None:
        dx, dgf = rmsnorm_bwd(dxf, x, gf, rstd)
    else:
        dx, dgf = dxf, None
    return loss, dx, dWv, dgf
