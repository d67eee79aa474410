"""The paper's analytic byte / FLOP model of one transformer layer (test infrastructure).

Symbols as in the paper's appendix: s sequence length, b micro-batch, h hidden, a query heads,
k kv heads, m FFN width, E experts, E_act active experts.  These closed forms assume a*d = h.
"""


def activation_bytes_per_layer(s, b, h, m, a, k, e_act=1):
    """App. B.1, Eq. act-mem: (12 + 4k/a) s b h + 6 s b m E_act bytes in a 16-bit format."""
    return (12.0 + 4.0 * k / a) * s * b * h + 6.0 * s * b * m * e_act


def checkpoint_bytes_per_layer(s, b, h):
    """Sec. 2.1.1: with full recomputation only the layer input is kept, 2 s b h bytes."""
    return 2.0 * s * b * h


def fwd_flops(s, b, h, m, a, k, e_act=1):
    """App. B.2, Eq. flops-dense.  The attention term is printed with the exponent on b; it has to be
    quadratic in the sequence length (QK^T and PV, non-causal), i.e. 4 s^2 b h."""
    return 4.0 * s * b * h * h + 4.0 * s * b * h * h * k / a + 4.0 * s * s * b * h + 6.0 * s * b * h * m * e_act


def fwd_upload_bytes(s, b, h, m, a, k, e=1):
    """App. C.1 / C.2, Eq. bytes-dense and its MoE variant: 4h^2 + 4h^2 k/a + 6 h m E + 2 b s h."""
    return 4.0 * h * h + 4.0 * h * h * k / a + 6.0 * h * m * e + 2.0 * b * s * h


def oi_fwd(s, b, h, m, a, k, e_act=1, e=1):
    """App. C.1 / C.2, Eq. oi-dense / oi-moe: forward FLOPs per uploaded byte."""
    return fwd_flops(s, b, h, m, a, k, e_act) / fwd_upload_bytes(s, b, h, m, a, k, e)


def bwd_flops(s, b, h, m, a, k, e_act=1):
    """App. C.3: recompute + activation gradient + weight gradient, each about one forward."""
    return 3.0 * fwd_flops(s, b, h, m, a, k, e_act)


def bubble_ratio_roundpipe(n_gpus, n_microbatches, n_stages):
    """Sec. 3.3: N(N-1) / (M S + N(N-1))."""
    n = n_gpus
    return n * (n - 1) / (n_microbatches * n_stages + n * (n - 1))
