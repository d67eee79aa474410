"""Thin harness around the binding: packs per-tensor arrays into the library's weight blob, owns the torch buffers
(device memory, pinned host memory, streams) and unpacks gradient blobs.  Marshalling only -- no layer math here.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from . import binding as B

_W_MAP = {"g1": "G1", "gq": "GQ", "gk": "GK", "Wo": "WO", "g2": "G2", "Wd": "WD"}
_LA = {"q": "LA_Q", "k": "LA_K", "v": "LA_V", "o": "LA_O", "gate": "LA_GATE", "up": "LA_UP", "down": "LA_DOWN"}
_LB = {"q": "LB_Q", "k": "LB_K", "v": "LB_V", "o": "LB_O", "gate": "LB_GATE", "up": "LB_UP", "down": "LB_DOWN"}


def f32_to_bf16_bits(a):
    """float32 ndarray whose values are bf16-representable (or not: round-to-nearest-even) -> uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)).astype(np.uint16)


def cfg_from_dict(c, with_head=None, n_layers=None):
    """Builds the library's stage configuration from a plain dict of shape numbers."""
    vocab = c["vocab"] if (with_head is None or with_head) else 0
    return B.make_cfg(n_layers=c["n_layers"] if n_layers is None else n_layers, hidden=c["hidden"],
                      n_q_heads=c["n_q_heads"], n_kv_heads=c["n_kv_heads"], head_dim=c["head_dim"], ffn=c["ffn"],
                      vocab=vocab, n_experts=c["n_experts"], top_k=c["top_k"], rope_base=c.get("rope_base", 1.0e6),
                      rms_eps=c.get("rms_eps", 1.0e-6), qk_norm=c.get("qk_norm", 1), lora_rank=c["lora_rank"],
                      lora_scale=c.get("lora_scale", 1.0), lora=c["lora"], train_base=c["train_base"],
                      moe_router=c.get("moe_router", 0), head_chunk=c.get("head_chunk", 0),
                      head_two_sweeps=c.get("head_two_sweeps", 0))


def _layer_tensors(p, cfg):
    """name -> list of ndarrays whose concatenation (flattened, in order) is the tensor in the library's fused order."""
    out = {"G1": [p["g1"]], "WQKV": [p["Wq"], p["Wk"], p["Wv"]], "WO": [p["Wo"]], "G2": [p["g2"]], "WD": [p["Wd"]]}
    if cfg.qk_norm:
        out["GQ"], out["GK"] = [p["gq"]], [p["gk"]]
    if cfg.n_experts > 0:
        # [E, 2m, h]: per expert the gate rows, then the up rows
        out["WGU"] = [a for e in range(cfg.n_experts) for a in (p["Wg"][e], p["Wu"][e])]
        if cfg.moe_router:
            out["WR"] = [p["Wr"]]
    else:
        out["WGU"] = [p["Wg"], p["Wu"]]                               # [2m, h]
    for name, (A, Bm) in p.get("lora", {}).items():
        out[_LA[name]], out[_LB[name]] = [A], [Bm]
    return out


_PACK_CHUNK = 1 << 22


def _store_bf16(dst16, arr):
    """dst16 (uint16 view of the blob) <- bf16 bits of arr, converted chunk by chunk on several threads."""
    flat = np.ascontiguousarray(arr, dtype=np.float32).reshape(-1)
    n = flat.size
    if n <= _PACK_CHUNK:
        dst16[:n] = f32_to_bf16_bits(flat)
        return
    def conv(i):
        dst16[i:i + _PACK_CHUNK] = f32_to_bf16_bits(flat[i:i + _PACK_CHUNK])
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(conv, range(0, n, _PACK_CHUNK)))


def pack_weights(cfg, layers, head=None, out=None):
    """Writes every tensor at the offset rp_weight_layout reports.  Returns a uint8 ndarray (the host blob)."""
    wbytes, _, _ = B.rp_query_sizes(cfg, 1, 8)
    blob = np.zeros(wbytes, dtype=np.uint8) if out is None else out
    b16 = blob.view(np.uint16)

    def put(layer, name, parts):
        off, n = B.rp_weight_layout(cfg, layer, B.T[name])
        if n == 0:
            return
        assert sum(a.size for a in parts) == n, (name, [a.shape for a in parts], n)
        pos = off // 2
        for a in parts:
            _store_bf16(b16[pos:pos + a.size], a)
            pos += a.size

    for li, p in enumerate(layers):
        for name, parts in _layer_tensors(p, cfg).items():
            put(li, name, parts)
    if head is not None and cfg.vocab > 0:
        put(cfg.n_layers, "GF", [head["gf"]])
        put(cfg.n_layers, "WV", [head["Wv"]])
    return blob


def unpack_grads(cfg, gblob):
    """fp32 gradient blob (torch tensor or ndarray of float32) -> list of per-layer dicts in the oracle's naming, head dict."""
    g = gblob.detach().cpu().numpy() if isinstance(gblob, torch.Tensor) else gblob
    g = g.view(np.float32)
    h, d = cfg.hidden, cfg.head_dim
    qd, kd, m, r = cfg.n_q_heads * d, cfg.n_kv_heads * d, cfg.ffn, cfg.lora_rank

    def get(layer, name, shape):
        off, n = B.rp_grad_layout(cfg, layer, B.T[name])
        if n == 0:
            return None
        return g[off // 4: off // 4 + n].reshape(shape).copy()

    layers = []
    for li in range(cfg.n_layers):
        o = {"lora": {}}
        wqkv = get(li, "WQKV", (qd + 2 * kd, h))
        if wqkv is not None:
            o["Wq"], o["Wk"], o["Wv"] = wqkv[:qd], wqkv[qd:qd + kd], wqkv[qd + kd:]
            wgu = get(li, "WGU", (2 * m, h))
            o["Wg"], o["Wu"] = wgu[:m], wgu[m:]
            o["Wo"], o["Wd"] = get(li, "WO", (h, qd)), get(li, "WD", (h, m))
            o["g1"], o["g2"] = get(li, "G1", (h,)), get(li, "G2", (h,))
            if cfg.qk_norm:
                o["gq"], o["gk"] = get(li, "GQ", (d,)), get(li, "GK", (d,))
        dims = {"q": (qd, h), "k": (kd, h), "v": (kd, h), "o": (h, qd), "gate": (m, h), "up": (m, h), "down": (h, m)}
        for name, (outd, ind) in dims.items():
            A = get(li, _LA[name], (r, ind))
            if A is not None:
                o["lora"][name] = (A, get(li, _LB[name], (outd, r)))
        layers.append(o)
    head = {}
    if cfg.vocab > 0:
        wv = get(cfg.n_layers, "WV", (cfg.vocab, h))
        if wv is not None:
            head = {"Wv": wv, "gf": get(cfg.n_layers, "GF", (h,))}
    return layers, head


def bf16_tensor(arr, device):
    """float32 ndarray -> torch bf16 tensor on device holding the RNE-rounded values."""
    bits = torch.from_numpy(f32_to_bf16_bits(arr).view(np.int16).reshape(arr.shape))
    return bits.to(device).view(torch.bfloat16)


def to_f32(t):
    return t.detach().float().cpu().numpy()


class StageRunner:
    """Owns a context, two streams, device slots, workspace and gradient blob for one stage shape."""

    def __init__(self, cfg, batch, seq, device="cuda:0", n_slots=1):
        self.cfg, self.batch, self.seq = cfg, batch, seq
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.compute = torch.cuda.Stream(device=self.device)
        self.copy = torch.cuda.Stream(device=self.device)
        self.wbytes, self.gbytes, self.wsbytes = B.rp_query_sizes(cfg, batch, seq)
        self.ctx = B.rp_ctx_create(self.device.index or 0, self.compute.cuda_stream, self.copy.cuda_stream, cfg)
        self.slot_bytes = B.rp_slot_bytes(cfg)      # the blob plus the tensors the library derives from it
        self.slots = [torch.empty(self.slot_bytes, dtype=torch.uint8, device=self.device) for _ in range(n_slots)]
        self.ws = torch.empty(self.wsbytes, dtype=torch.uint8, device=self.device)
        # the head gets a workspace of its own so that it can run between the two phases of a fused last stage
        self.ws_head = self.ws
        if cfg.vocab > 0 and cfg.n_layers > 0:
            self.ws_head = torch.empty(self.wsbytes, dtype=torch.uint8, device=self.device)
        self.grads = torch.zeros(max(self.gbytes, 4) // 4, dtype=torch.float32, device=self.device)
        self.T = batch * seq

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize(self.device)
            B.rp_ctx_destroy(self.ctx)
            self.ctx = None

    def pinned_blob(self, layers, head=None):
        host = torch.empty(self.wbytes, dtype=torch.uint8, pin_memory=True)
        pack_weights(self.cfg, layers, head, out=host.numpy())
        return host

    def upload(self, host_blob, slot=0):
        B.rp_stage_upload_weights(self.ctx, slot, self.slots[slot], host_blob, self.wbytes)

    def bind(self, slot=0):
        B.rp_stage_bind_weights(self.ctx, slot, self.slots[slot], self.wbytes)

    def forward(self, x, slot=0, keep_layer_inputs=False, router=None):
        """router: fp32 device tensor [n_layers, T, E] of router logits (MoE stages): input, or with cfg.moe_router the
        buffer that receives the logits the stage computes."""
        out = torch.empty_like(x)
        keep = None
        if keep_layer_inputs:
            keep = [torch.empty_like(x) for _ in range(self.cfg.n_layers)]
        B.rp_stage_forward(self.ctx, slot, x, out, keep, router, self.batch, self.seq, self.ws, self.wsbytes)
        return (out, keep) if keep_layer_inputs else out

    def backward(self, x, dy, slot=0, want_out=True, router=None, d_router=None):
        """Ordinary backward stage: recomputation followed by the backward pass."""
        dx = torch.empty_like(x)
        out = torch.empty_like(x) if want_out else None
        B.rp_stage_backward(self.ctx, slot, B.PHASE_BOTH, x, dy, dx, out, self.grads if self.gbytes else None, router,
                            d_router, self.batch, self.seq, self.ws, self.wsbytes)
        return out, dx

    def recompute(self, x, out, slot=0):
        """First half of the fused last stage: forward keeping the internals in the workspace."""
        B.rp_stage_backward(self.ctx, slot, B.PHASE_RECOMPUTE, x, None, None, out, None, None, None, self.batch, self.seq,
                            self.ws, self.wsbytes)

    def backward_only(self, x, dy, dx, slot=0):
        """Second half: backward from the internals the recompute phase left in the workspace."""
        B.rp_stage_backward(self.ctx, slot, B.PHASE_BACKWARD, x, dy, dx, None, self.grads if self.gbytes else None, None,
                            None, self.batch, self.seq, self.ws, self.wsbytes)

    def fused_last_stage(self, x, labels, out, dy_head, dx, loss, grad_scale=1.0, slot=0, train=True):
        """The fused last stage (paper Sec. 3.2: its forward doubles as the recomputation), as three calls on caller-
        owned buffers: forward keeping the internals -> LM head + loss on its own workspace (dy_head receives the
        gradient of the stage output) -> backward from the kept internals.  This is the step bench.py times."""
        self.recompute(x, out, slot)
        self.head(out, labels, grad_scale, slot, train=train, loss=loss, dx=dy_head)
        self.backward_only(x, dy_head, dx, slot)
        return loss

    def head(self, x, labels, grad_scale=1.0, slot=0, train=True, loss=None, dx=None):
        if loss is None:
            loss = torch.empty(1, dtype=torch.float32, device=self.device)
        if dx is None:
            dx = torch.empty_like(x)
        B.rp_lmhead_ce_fwd_bwd(self.ctx, slot, x, labels, loss, dx, self.grads if (train and self.gbytes) else None,
                               grad_scale, self.batch, self.seq, self.ws_head, self.wsbytes)
        return loss, dx

    def enable_rounds(self, streams_per_direction=1):
        """Sets up the transfer streams of the multi-stream worker.  streams_per_direction = 2: activations and
        parameters / gradients on streams of their own (five streams with compute, as in the paper); 1: one stream per
        direction -- activation uploads share the parameter-upload stream, gradient downloads the activation-download
        stream -- which keeps the process within the runtime's default of four hardware queues."""
        self.act_down = torch.cuda.Stream(device=self.device)
        if streams_per_direction == 2:
            self.act_up = torch.cuda.Stream(device=self.device)
            self.grad_down = torch.cuda.Stream(device=self.device)
        else:
            self.act_up, self.grad_down = self.copy, self.act_down
        B.rp_ctx_set_transfer_streams(self.ctx, self.act_up.cuda_stream, self.act_down.cuda_stream, self.grad_down.cuda_stream)
        shape = (self.T, self.cfg.hidden)
        mk = lambda: [torch.empty(shape, dtype=torch.bfloat16, device=self.device) for _ in range(2)]
        self.x_stage, self.dy_stage, self.out_stage = mk(), mk(), mk()

    def round(self, x_host, out_host, slot=0, dy_host=None, next_slot=-1, next_host_blob=None, done_grads_dev=None,
              done_grads_host=None, max_piece_bytes=0):
        """One stage over len(x_host) micro-batches with host-resident activations; backward round when dy_host is given."""
        io = B.make_round_io(x_host, out_host, self.x_stage, self.out_stage, dy_host, self.dy_stage if dy_host is not None else None,
                             next_slot, self.slots[next_slot] if next_slot >= 0 else None, next_host_blob, done_grads_dev,
                             done_grads_host, max_piece_bytes)
        if dy_host is None:
            B.rp_round_forward(self.ctx, slot, io, self.batch, self.seq, self.ws, self.wsbytes)
        else:
            B.rp_round_backward(self.ctx, slot, io, self.grads if self.gbytes else None, self.batch, self.seq, self.ws, self.wsbytes)
        return io

    def sync(self):
        self.compute.synchronize()
        self.copy.synchronize()
        for name in ("act_up", "act_down", "grad_down"):
            if hasattr(self, name):
                getattr(self, name).synchronize()
