"""Pins of the oracle's layer functions against things other than itself: central finite
differences, closed forms, invariants and brute-force loops (all fp64, tiny shapes)."""
import math

import numpy as np
import pytest

from oracle import layers as L

RNG = np.random.default_rng(1234)


def fd_check(f, arrays, analytic, n_probe=12, eps=1e-6, tol=2e-6):
    """f() -> scalar, reading the arrays in `arrays` (perturbed in place).  analytic[i] is d f / d arrays[i]."""
    for arr, an in zip(arrays, analytic):
        flat = arr.reshape(-1)
        an_flat = np.asarray(an).reshape(-1)
        assert flat.shape == an_flat.shape
        idx = RNG.choice(flat.size, size=min(n_probe, flat.size), replace=False)
        scale = max(np.max(np.abs(an_flat)), 1e-12)
        for i in idx:
            old = flat[i]
            flat[i] = old + eps
            fp = f()
            flat[i] = old - eps
            fm = f()
            flat[i] = old
            fd = (fp - fm) / (2 * eps)
            assert abs(fd - an_flat[i]) <= tol * scale + 1e-9, (i, fd, an_flat[i])


# ----------------------------------------------------------------------------- RMSNorm
def test_rmsnorm_unit_gain_mean_square():
    x = RNG.standard_normal((5, 16)) * 3.0
    eps = 1e-6
    y, rstd = L.rmsnorm_fwd(x, np.ones(16), eps)
    ms = np.mean(x * x, axis=-1)
    np.testing.assert_allclose(np.mean(y * y, axis=-1), ms / (ms + eps), rtol=1e-12)
    # element check against a python loop
    for t in range(5):
        r = 1.0 / math.sqrt(sum(float(v) ** 2 for v in x[t]) / 16 + eps)
        for j in range(16):
            assert abs(y[t, j] - x[t, j] * r) < 1e-12


def test_rmsnorm_scale_invariance():
    x = RNG.standard_normal((4, 8))
    g = RNG.standard_normal(8)
    y1, _ = L.rmsnorm_fwd(x, g, 0.0)
    y2, _ = L.rmsnorm_fwd(7.5 * x, g, 0.0)
    np.testing.assert_allclose(y1, y2, rtol=1e-12)


def test_rmsnorm_bwd_fd():
    x = RNG.standard_normal((6, 10))
    g = RNG.standard_normal(10)
    dy = RNG.standard_normal((6, 10))
    _, rstd = L.rmsnorm_fwd(x, g, 1e-6)
    dx, dg = L.rmsnorm_bwd(dy, x, g, rstd)
    fd_check(lambda: float(np.sum(dy * L.rmsnorm_fwd(x, g, 1e-6)[0])), [x, g], [dx, dg])


def test_rmsnorm_per_head_bwd_fd():
    x = RNG.standard_normal((3, 4, 6))
    g = RNG.standard_normal(6)
    dy = RNG.standard_normal((3, 4, 6))
    _, rstd = L.rmsnorm_fwd(x, g, 1e-6)
    dx, dg = L.rmsnorm_bwd(dy, x, g, rstd)
    fd_check(lambda: float(np.sum(dy * L.rmsnorm_fwd(x, g, 1e-6)[0])), [x, g], [dx, dg])


# ----------------------------------------------------------------------------- Linear + LoRA
def test_linear_matches_loops():
    u = RNG.standard_normal((3, 5))
    W = RNG.standard_normal((4, 5))
    y = L.linear_fwd(u, W)
    for t in range(3):
        for o in range(4):
            assert abs(y[t, o] - sum(u[t, i] * W[o, i] for i in range(5))) < 1e-12


def test_lora_zero_B_is_base_and_dA_zero():
    u = RNG.standard_normal((7, 6))
    W = RNG.standard_normal((5, 6))
    A = RNG.standard_normal((2, 6))
    B = np.zeros((5, 2))
    np.testing.assert_array_equal(L.linear_fwd(u, W, (A, B), 0.7), L.linear_fwd(u, W))
    dy = RNG.standard_normal((7, 5))
    du, dW, dA, dB = L.linear_bwd(dy, u, W, (A, B), 0.7)
    assert np.all(dA == 0.0)
    assert np.any(dB != 0.0)
    np.testing.assert_allclose(du, dy @ W, rtol=1e-12)


def test_lora_merged_weight_identity():
    u = RNG.standard_normal((7, 6))
    W = RNG.standard_normal((5, 6))
    A = RNG.standard_normal((2, 6))
    B = RNG.standard_normal((5, 2))
    s = 1.7
    np.testing.assert_allclose(L.linear_fwd(u, W, (A, B), s), u @ (W + s * B @ A).T, rtol=1e-11, atol=1e-12)


def test_linear_lora_bwd_fd():
    u = RNG.standard_normal((7, 6))
    W = RNG.standard_normal((5, 6))
    A = RNG.standard_normal((2, 6))
    B = RNG.standard_normal((5, 2))
    dy = RNG.standard_normal((7, 5))
    s = 0.6
    du, dW, dA, dB = L.linear_bwd(dy, u, W, (A, B), s)
    fd_check(lambda: float(np.sum(dy * L.linear_fwd(u, W, (A, B), s))), [u, W, A, B], [du, dW, dA, dB])


# ----------------------------------------------------------------------------- RoPE
def test_rope_properties():
    batch, seq, H, d = 2, 9, 3, 8
    u = RNG.standard_normal((batch * seq, H, d))
    r = L.rope_fwd(u, batch, seq, 1.0e4)
    # rotation: norms of each (i, i+d/2) pair preserved
    n0 = u[..., : d // 2] ** 2 + u[..., d // 2:] ** 2
    n1 = r[..., : d // 2] ** 2 + r[..., d // 2:] ** 2
    np.testing.assert_allclose(n0, n1, rtol=1e-12)
    # position 0 of every sequence is the identity
    for bi in range(batch):
        np.testing.assert_allclose(r[bi * seq], u[bi * seq], rtol=0, atol=1e-15)
    # backward is the inverse rotation
    np.testing.assert_allclose(L.rope_bwd(r, batch, seq, 1.0e4), u, rtol=1e-12, atol=1e-13)


def test_rope_explicit_angle():
    # one vector, position 3, pair i=1 of d=4: angle 3 * base^(-2/4)
    base = 100.0
    u = np.zeros((4, 1, 4))
    u[3, 0, :] = [0.0, 1.0, 0.0, 0.0]
    r = L.rope_fwd(u, 1, 4, base)
    phi = 3 * base ** (-0.5)
    np.testing.assert_allclose(r[3, 0], [0.0, math.cos(phi), 0.0, math.sin(phi)], atol=1e-14)


def test_rope_relative_position():
    d, base = 8, 50.0
    q = RNG.standard_normal(d)
    k = RNG.standard_normal(d)
    seq = 12

    def dot(p, pp):
        U = np.zeros((seq, 2, d))
        U[p, 0] = q
        U[pp, 1] = k
        R = L.rope_fwd(U, 1, seq, base)
        return float(R[p, 0] @ R[pp, 1])

    assert abs(dot(7, 3) - dot(9, 5)) < 1e-12
    assert abs(dot(4, 4) - float(q @ k)) < 1e-12
    assert abs(dot(7, 3) - dot(7, 4)) > 1e-6


def test_rope_bwd_fd():
    batch, seq, H, d = 2, 5, 2, 6
    u = RNG.standard_normal((batch * seq, H, d))
    dy = RNG.standard_normal(u.shape)
    du = L.rope_bwd(dy, batch, seq, 1.0e3)
    fd_check(lambda: float(np.sum(dy * L.rope_fwd(u, batch, seq, 1.0e3))), [u], [du])


# ----------------------------------------------------------------------------- attention
def brute_attention(q, k, v, batch, seq):
    """Pure-python causal GQA attention, one score at a time."""
    T, a, d = q.shape
    kh = k.shape[1]
    o = np.zeros_like(q)
    for bi in range(batch):
        for j in range(a):
            g = j // (a // kh)
            for t in range(seq):
                sc = [sum(q[bi * seq + t, j, e] * k[bi * seq + u, g, e] for e in range(d)) / math.sqrt(d)
                      for u in range(t + 1)]
                mx = max(sc)
                w = [math.exp(x - mx) for x in sc]
                z = sum(w)
                for u in range(t + 1):
                    o[bi * seq + t, j] += (w[u] / z) * v[bi * seq + u, g]
    return o


def test_attention_vs_brute_force_gqa():
    batch, seq, a, kh, d = 2, 7, 4, 2, 4
    q = RNG.standard_normal((batch * seq, a, d))
    k = RNG.standard_normal((batch * seq, kh, d))
    v = RNG.standard_normal((batch * seq, kh, d))
    o, P, lse = L.attention_fwd(q, k, v, batch, seq)
    np.testing.assert_allclose(o, brute_attention(q, k, v, batch, seq), rtol=1e-11, atol=1e-12)
    for row in P:
        for Pm in row:
            np.testing.assert_allclose(Pm.sum(axis=-1), 1.0, rtol=1e-12)
            assert np.all(np.triu(Pm, k=1) == 0.0)


def test_attention_causality_and_special_cases():
    batch, seq, a, kh, d = 1, 10, 2, 1, 4
    q = RNG.standard_normal((seq, a, d))
    k = RNG.standard_normal((seq, kh, d))
    v = RNG.standard_normal((seq, kh, d))
    o, _, _ = L.attention_fwd(q, k, v, batch, seq)
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[6:] += 5.0
    v2[6:] -= 3.0
    q2[6:] *= 2.0
    o2, _, _ = L.attention_fwd(q2, k2, v2, batch, seq)
    np.testing.assert_array_equal(o[:6], o2[:6])          # outputs before position 6 untouched
    # zero queries -> uniform weights -> running mean of v
    o3, _, lse3 = L.attention_fwd(np.zeros_like(q), k, v, batch, seq)
    for t in range(seq):
        np.testing.assert_allclose(o3[t, 0], v[: t + 1, 0].mean(axis=0), rtol=1e-12)
        assert abs(lse3[0, 0, t] - math.log(t + 1)) < 1e-12
    # seq = 1 -> o = v
    o4, _, _ = L.attention_fwd(q[:1], k[:1], v[:1], 1, 1)
    np.testing.assert_allclose(o4[0, 0], v[0, 0], rtol=1e-14)
    np.testing.assert_allclose(o4[0, 1], v[0, 0], rtol=1e-14)


def test_attention_bwd_fd():
    batch, seq, a, kh, d = 2, 6, 4, 2, 4
    q = RNG.standard_normal((batch * seq, a, d))
    k = RNG.standard_normal((batch * seq, kh, d))
    v = RNG.standard_normal((batch * seq, kh, d))
    do = RNG.standard_normal(q.shape)
    o, P, _ = L.attention_fwd(q, k, v, batch, seq)
    dq, dk, dv = L.attention_bwd(do, q, k, v, o, P, batch, seq)
    fd_check(lambda: float(np.sum(do * L.attention_fwd(q, k, v, batch, seq)[0])), [q, k, v], [dq, dk, dv],
             n_probe=20)


# ----------------------------------------------------------------------------- SwiGLU
def test_swiglu_values_and_fd():
    g = np.array([[0.0, 1.0, -2.0]])
    u = np.array([[3.0, 2.0, 0.5]])
    act = L.swiglu_fwd(g, u)
    np.testing.assert_allclose(act[0], [0.0, 2.0 / (1 + math.exp(-1.0)), -2.0 * 0.5 / (1 + math.exp(2.0))],
                               rtol=1e-14)
    g = RNG.standard_normal((4, 5))
    u = RNG.standard_normal((4, 5))
    d = RNG.standard_normal((4, 5))
    dg, du = L.swiglu_bwd(d, g, u)
    fd_check(lambda: float(np.sum(d * L.swiglu_fwd(g, u))), [g, u], [dg, du])


# ----------------------------------------------------------------------------- MoE
def dense_ffn(n2, Wg, Wu, Wd):
    return L.swiglu_fwd(n2 @ Wg.T, n2 @ Wu.T) @ Wd.T


def test_moe_single_expert_is_dense():
    T, h, m = 5, 6, 7
    n2 = RNG.standard_normal((T, h))
    Wg, Wu, Wd = RNG.standard_normal((1, m, h)), RNG.standard_normal((1, m, h)), RNG.standard_normal((1, h, m))
    out, _ = L.moe_ffn_fwd(n2, Wg, Wu, Wd, RNG.standard_normal((T, 1)), 1)
    np.testing.assert_allclose(out, dense_ffn(n2, Wg[0], Wu[0], Wd[0]), rtol=1e-12, atol=1e-12)


def test_moe_all_experts_is_softmax_mixture():
    T, h, m, E = 4, 5, 6, 3
    n2 = RNG.standard_normal((T, h))
    Wg, Wu, Wd = RNG.standard_normal((E, m, h)), RNG.standard_normal((E, m, h)), RNG.standard_normal((E, h, m))
    logits = RNG.standard_normal((T, E))
    out, _ = L.moe_ffn_fwd(n2, Wg, Wu, Wd, logits, E)
    p = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
    ref = sum(p[:, e:e + 1] * dense_ffn(n2, Wg[e], Wu[e], Wd[e]) for e in range(E))
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)


def test_moe_route_topk_and_renormalised_softmax_agree():
    T, E, K = 50, 16, 4
    logits = RNG.standard_normal((T, E))
    idx, w = L.moe_route(logits, K)
    p = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
    for t in range(T):
        top = sorted(range(E), key=lambda e: (-logits[t, e], e))[:K]
        assert list(idx[t]) == top
        sel = p[t, top] / p[t, top].sum()
        np.testing.assert_allclose(w[t], sel, rtol=1e-12)
    np.testing.assert_allclose(w.sum(-1), 1.0, rtol=1e-12)


def test_moe_route_ties_prefer_lower_index():
    logits = np.array([[1.0, 2.0, 2.0, 0.0, 2.0]])
    idx, w = L.moe_route(logits, 2)
    assert list(idx[0]) == [1, 2]
    np.testing.assert_allclose(w[0], [0.5, 0.5])


def test_moe_bwd_fd():
    T, h, m, E, K = 4, 5, 6, 5, 2
    n2 = RNG.standard_normal((T, h))
    Wg, Wu, Wd = RNG.standard_normal((E, m, h)), RNG.standard_normal((E, m, h)), RNG.standard_normal((E, h, m))
    logits = RNG.standard_normal((T, E)) * 2.0
    dout = RNG.standard_normal((T, h))
    out, rc = L.moe_ffn_fwd(n2, Wg, Wu, Wd, logits, K)
    dn2, dlog, (dWg, dWu, dWd) = L.moe_ffn_bwd(dout, n2, Wg, Wu, Wd, rc, want_dW=True)
    fd_check(lambda: float(np.sum(dout * L.moe_ffn_fwd(n2, Wg, Wu, Wd, logits, K)[0])),
             [n2, logits, Wg, Wu, Wd], [dn2, dlog, dWg, dWu, dWd], n_probe=20)


# ----------------------------------------------------------------------------- LM head + CE
def test_ce_brute_force_per_row():
    T, h, V = 6, 5, 11
    x = RNG.standard_normal((T, h))
    Wv = RNG.standard_normal((V, h))
    labels = np.array([3, 0, -100, 10, 7, -100], dtype=np.int32)
    loss, dx, dW, _ = L.lmhead_ce_fwd_bwd(x, Wv, labels)
    tot, n = 0.0, 0
    for t in range(T):
        if labels[t] == -100:
            continue
        z = [sum(x[t, i] * Wv[vv, i] for i in range(h)) for vv in range(V)]
        tot += -math.log(math.exp(z[labels[t]]) / sum(math.exp(zz) for zz in z))
        n += 1
    assert abs(loss - tot / n) < 1e-12
    assert np.all(dx[2] == 0.0) and np.all(dx[5] == 0.0)


def test_ce_uniform_logits_closed_form():
    for V in (4096, 151936):
        x = np.zeros((2, 3))
        Wv = RNG.standard_normal((V, 3))
        loss, dx, _, _ = L.lmhead_ce_fwd_bwd(x, Wv, np.array([1, V - 1], dtype=np.int32), want_dW=False)
        assert abs(loss - math.log(V)) < 1e-12
    assert abs(math.log(4096) - 8.31777) < 1e-5 and abs(math.log(151936) - 11.93121) < 1e-5


def test_ce_dz_rows_sum_to_zero():
    # identical rows in Wv: dx_t = (sum_v dZ_tv) * w = 0
    T, h, V = 4, 5, 9
    x = RNG.standard_normal((T, h))
    Wv = np.tile(RNG.standard_normal((1, h)), (V, 1))
    _, dx, dW, _ = L.lmhead_ce_fwd_bwd(x, Wv, np.array([0, 1, 2, 3], dtype=np.int32))
    np.testing.assert_allclose(dx, 0.0, atol=1e-14)
    np.testing.assert_allclose(dW.sum(axis=0), 0.0, atol=1e-13)


def test_ce_chunked_equals_unchunked():
    T, h, V = 5, 4, 23
    x = RNG.standard_normal((T, h))
    Wv = RNG.standard_normal((V, h))
    labels = np.array([0, 22, 5, -100, 9], dtype=np.int32)
    loss, _, _, _ = L.lmhead_ce_fwd_bwd(x, Wv, labels)
    # online (max, sum) over vocab chunks of 7
    m = np.full(T, -np.inf)
    s = np.zeros(T)
    for c0 in range(0, V, 7):
        Z = x @ Wv[c0:c0 + 7].T
        mn = np.maximum(m, Z.max(-1))
        s = s * np.exp(m - mn) + np.exp(Z - mn[:, None]).sum(-1)
        m = mn
    lse = m + np.log(s)
    valid = labels != -100
    ref = np.mean([lse[t] - x[t] @ Wv[labels[t]] for t in range(T) if valid[t]])
    assert abs(loss - ref) < 1e-12


def test_ce_bwd_fd_with_final_norm_and_scale():
    T, h, V = 5, 6, 13
    x = RNG.standard_normal((T, h))
    Wv = RNG.standard_normal((V, h))
    gf = RNG.standard_normal(h)
    labels = np.array([1, -100, 12, 4, 0], dtype=np.int32)
    gs = 3.0
    loss, dx, dW, dgf = L.lmhead_ce_fwd_bwd(x, Wv, labels, gf, 1e-6, gs)
    fd_check(lambda: gs * L.lmhead_ce_fwd_bwd(x, Wv, labels, gf, 1e-6, 1.0, want_dW=False)[0],
             [x, Wv, gf], [dx, dW, dgf], n_probe=20)
