"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU harness.

Data only: this module draws random numbers, rounds them to bf16 (round-to-nearest-even, by bit
arithmetic) and names the workload shapes.  It contains none of the method's arithmetic and imports
neither the oracle nor the HIP package.

The workloads are the synthetic stage configurations this build is measured on (shapes after the
paper's Table "Model Configs": five Qwen3-shaped ones and a GPT-OSS-20B-shaped mixture of experts
whose router is part of the layer); weights N(0, 0.02), LoRA A N(0, 0.02), LoRA B N(0, 0.01), norm
gains 1, token ids uniform, labels = next token.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

SEED_BASE = 27085
LORA_ORDER = ("q", "k", "v", "o", "gate", "up", "down")

# name -> plain numbers.  'lora' lists the adapted projections; 'stream' marks host-streamed frozen bases.
CONFIGS = {
    "C1": dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=688, vocab=4096,
               n_experts=0, top_k=0, lora_rank=8, lora=("q", "v"), train_base=1, batch=1, seq=128,
               x_from="emb", stream=0),
    "C2": dict(n_layers=4, hidden=2048, n_q_heads=16, n_kv_heads=8, head_dim=128, ffn=6144, vocab=151936,
               n_experts=0, top_k=0, lora_rank=0, lora=(), train_base=1, batch=1, seq=4096,
               x_from="emb", stream=0),
    "C3": dict(n_layers=4, hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=12288, vocab=0,
               n_experts=0, top_k=0, lora_rank=16, lora=LORA_ORDER, train_base=0, batch=1, seq=8192,
               x_from="normal", stream=1),
    "C4": dict(n_layers=2, hidden=5120, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=25600, vocab=151936,
               n_experts=0, top_k=0, lora_rank=16, lora=LORA_ORDER, train_base=0, batch=1, seq=16384,
               x_from="normal", stream=1),
    "C5": dict(n_layers=1, hidden=4096, n_q_heads=64, n_kv_heads=4, head_dim=128, ffn=1536, vocab=0,
               n_experts=128, top_k=8, lora_rank=8, lora=("q", "k", "v", "o"), train_base=0, batch=1,
               seq=31744, x_from="normal", stream=1),
    # GPT-OSS-20B row of the table: h = m = 2880 (not a multiple of the 256-wide GEMM tiles), 4 of 32 experts,
    # router weights in the layer
    "C6": dict(n_layers=4, hidden=2880, n_q_heads=64, n_kv_heads=8, head_dim=64, ffn=2880, vocab=0,
               n_experts=32, top_k=4, lora_rank=8, lora=("q", "k", "v", "o"), train_base=0, batch=1,
               seq=8192, x_from="normal", stream=1, moe_router=1),
}
ROPE_BASE = 1.0e6
RMS_EPS = 1.0e-6


def config_seed(name):
    return SEED_BASE + sorted(CONFIGS).index(name)


# ----------------------------------------------------------------------------- bf16 helpers (bit arithmetic only)
def bf16_bits(x):
    """float32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even (NaN kept quiet)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if np.any(nan):
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bits_to_f32(b):
    """uint16 bf16 bit patterns -> float32 array holding exactly those values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x):
    """float32 array -> float32 array whose values are exactly representable in bf16."""
    return bits_to_f32(bf16_bits(x)).reshape(np.shape(x))


_PAR_CHUNK = 1 << 22      # elements per independently drawn chunk of a large tensor


def _normal(rng, shape, std):
    """N(0, std) rounded to bf16.  Tensors of more than one chunk are drawn chunk by chunk from child generators spawned
    off rng (a fixed function of the seed and the shape, whatever the number of threads), several chunks at a time:
    the larger workloads hold billions of parameters."""
    n = int(np.prod(shape))
    if n <= _PAR_CHUNK:
        return bf16_round(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))
    out = np.empty(n, dtype=np.float32)
    nchunk = -(-n // _PAR_CHUNK)
    kids = rng.spawn(nchunk)

    def fill(i):
        sl = out[i * _PAR_CHUNK:(i + 1) * _PAR_CHUNK]
        kids[i].standard_normal(out=sl, dtype=np.float32)
        sl *= np.float32(std)
        u = sl.view(np.uint32)                       # round to nearest even in place (no NaN among normal draws)
        u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        u &= np.uint32(0xFFFF0000)

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(fill, range(nchunk)))
    return out.reshape(shape)


# ----------------------------------------------------------------------------- parameter / input draws
def make_layer(rng, c, gains_random=False):
    """One layer's parameters as float32 arrays holding bf16-representable values."""
    h, d = c["hidden"], c["head_dim"]
    qd, kd, m, E = c["n_q_heads"] * d, c["n_kv_heads"] * d, c["ffn"], c["n_experts"]
    gain = (lambda n: bf16_round(1.0 + 0.1 * rng.standard_normal(n, dtype=np.float32))) if gains_random \
        else (lambda n: np.ones(n, dtype=np.float32))
    p = {"g1": gain(h), "Wq": _normal(rng, (qd, h), 0.02), "Wk": _normal(rng, (kd, h), 0.02),
         "Wv": _normal(rng, (kd, h), 0.02), "gq": gain(d), "gk": gain(d),
         "Wo": _normal(rng, (h, qd), 0.02), "g2": gain(h)}
    if E > 0:
        p["Wg"] = _normal(rng, (E, m, h), 0.02)
        p["Wu"] = _normal(rng, (E, m, h), 0.02)
        p["Wd"] = _normal(rng, (E, h, m), 0.02)
    else:
        p["Wg"] = _normal(rng, (m, h), 0.02)
        p["Wu"] = _normal(rng, (m, h), 0.02)
        p["Wd"] = _normal(rng, (h, m), 0.02)
    if E > 0 and c.get("moe_router"):
        p["Wr"] = _normal(rng, (E, h), 0.02)
    r = c["lora_rank"]
    p["lora"] = {}
    if r > 0:
        dims = {"q": (qd, h), "k": (kd, h), "v": (kd, h), "o": (h, qd), "gate": (m, h), "up": (m, h), "down": (h, m)}
        for name in LORA_ORDER:
            if name in c["lora"]:
                out, inn = dims[name]
                p["lora"][name] = (_normal(rng, (r, inn), 0.02), _normal(rng, (out, r), 0.01))
    return p


def make_head(rng, c, gains_random=False):
    h, V = c["hidden"], c["vocab"]
    gf = bf16_round(1.0 + 0.1 * rng.standard_normal(h, dtype=np.float32)) if gains_random \
        else np.ones(h, dtype=np.float32)
    return {"gf": gf, "Wv": _normal(rng, (V, h), 0.02)}


def make_workload(c, seed, gains_random=False, with_head=None):
    """Draws everything one stage call needs.  Returns a dict:
    layers (list of layer dicts), head (or None), x [T,h], dy [T,h], labels int32 [T] (or None),
    router_logits (list of fp32 [T,E] per layer; None for dense stages and for stages that hold their router)."""
    rng = np.random.default_rng(seed)
    T = c["batch"] * c["seq"]
    h = c["hidden"]
    layers = [make_layer(rng, c, gains_random) for _ in range(c["n_layers"])]
    if with_head is None:
        with_head = c["vocab"] > 0
    head = make_head(rng, c, gains_random) if with_head else None
    labels = None
    if c.get("x_from", "normal") == "emb" and c["vocab"] > 0:
        V = c["vocab"]
        ids = rng.integers(0, V, size=(c["batch"], c["seq"]), dtype=np.int64)
        emb = _normal(rng, (V, h), 0.02)
        x = emb[ids.reshape(-1)]
        lab = np.full((c["batch"], c["seq"]), -100, dtype=np.int32)
        lab[:, :-1] = ids[:, 1:]
        labels = lab.reshape(-1)
    else:
        x = _normal(rng, (T, h), 1.0)
        if c["vocab"] > 0:
            labels = rng.integers(0, c["vocab"], size=T, dtype=np.int64).astype(np.int32)
    dy = _normal(rng, (T, h), 1.0)
    router = None
    if c["n_experts"] > 0 and not c.get("moe_router"):      # else the layers hold a router and compute the logits
        router = [rng.standard_normal((T, c["n_experts"]), dtype=np.float32) for _ in range(c["n_layers"])]
    return dict(layers=layers, head=head, x=np.ascontiguousarray(x), dy=dy, labels=labels, router_logits=router)


def plant_routing(wl, c, seed, beta=0.25, level0=8.0, step=2.0, noise=0.002):
    """Rewrites a drawn workload so that every token has a decisive router preference (a trained router's logits are
    well separated; independent normal draws have near-ties that make the chosen expert set depend on the last bit).
    Token t gets top_k hidden coordinates set to the levels level0, level0+step, ...; layer l's router row of expert e
    is beta on coordinate perm_l[e] plus N(0, noise).  The residual stream carries the planted coordinates through the
    layers, so the gaps between the logits stay near beta*step/rms(x).  Data only: nothing here evaluates the layer."""
    rng = np.random.default_rng(seed + 7919)
    E, k, h = c["n_experts"], c["top_k"], c["hidden"]
    assert c.get("moe_router") and h >= E
    T = wl["x"].shape[0]
    x = wl["x"].copy()
    x[:, :E] = bf16_round(0.5 * x[:, :E])
    levels = (level0 + step * np.arange(k)).astype(np.float32)
    for t in range(T):
        x[t, rng.permutation(E)[:k]] = levels
    wl["x"] = bf16_round(x)
    for p in wl["layers"]:
        Wr = rng.standard_normal((E, h), dtype=np.float32) * np.float32(noise)
        perm = rng.permutation(E)
        Wr[np.arange(E), perm] = beta
        p["Wr"] = bf16_round(Wr)
    return wl


def shrink(c, **over):
    """A copy of a config dict with some numbers replaced (e.g. a shorter sequence for oracle-sized parity)."""
    d = dict(c)
    d.update(over)
    return d
