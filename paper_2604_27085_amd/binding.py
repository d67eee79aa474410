"""ctypes binding of librp.so: the same entry points as include/rp.h and include/rp_ops.h, argument marshalling only.

Every computation runs inside the HIP library.  There is no fallback: importing this module without a built
librp.so raises, and nothing here imports the CPU oracle.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librp.so")

RP_OK, RP_EINVAL, RP_ENOMEM, RP_EHIP, RP_ESTATE, RP_EUNSUPPORTED = range(6)
RP_MAX_SLOTS = 4
IGNORE_INDEX = -100
LORA_BITS = {"q": 1, "k": 2, "v": 4, "o": 8, "gate": 16, "up": 32, "down": 64}
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2
PHASE_RECOMPUTE, PHASE_BACKWARD, PHASE_BOTH = 1, 2, 3

TENSOR_IDS = ["G1", "WQKV", "GQ", "GK", "WO", "G2", "WGU", "WD", "WR", "LA_Q", "LA_K", "LA_V", "LB_Q", "LB_K", "LB_V",
              "LA_O", "LB_O", "LA_GATE", "LA_UP", "LB_GATE", "LB_UP", "LA_DOWN", "LB_DOWN", "GF", "WV"]
T = {name: i for i, name in enumerate(TENSOR_IDS)}


class StageCfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float),
                ("qk_norm", C.c_int32), ("lora_rank", C.c_int32), ("lora_scale", C.c_float), ("lora_mask", C.c_uint32),
                ("train_base", C.c_int32), ("moe_router", C.c_int32), ("head_chunk", C.c_int32), ("head_two_sweeps", C.c_int32)]


class Piece(C.Structure):
    _fields_ = [("item", C.c_int32), ("window", C.c_int32), ("offset", C.c_size_t), ("bytes", C.c_size_t)]


class RoundIO(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_micro", C.c_int32), ("x_host", C.POINTER(C.c_void_p)),
                ("dy_host", C.POINTER(C.c_void_p)), ("out_host", C.POINTER(C.c_void_p)), ("x_dev", C.c_void_p * 2),
                ("dy_dev", C.c_void_p * 2), ("out_dev", C.c_void_p * 2), ("next_slot", C.c_int32),
                ("next_dev_slot", C.c_void_p), ("next_host_blob", C.c_void_p), ("done_grads_dev", C.c_void_p),
                ("done_grads_host", C.c_void_p), ("max_piece_bytes", C.c_size_t)]


class TraceRecord(C.Structure):
    _fields_ = [("name", C.c_char * 40), ("flops", C.c_double), ("bytes", C.c_double), ("ms", C.c_float)]


class RpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("rp status %d: %s" % (code, msg))
        self.code = code


def _load():
    # PyTorch wheels bundle their own HIP runtime (same soname as the system one).  A process must talk to exactly one
    # runtime, or streams and events handed across the boundary belong to a different runtime than the one the
    # kernels are launched with: load torch's copy first so that librp.so binds to it.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise ImportError("librp.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2604_27085_amd/build.py) first; there is no CPU fallback")
    return C.CDLL(LIB_PATH)


lib = _load()

_vp, _i, _l, _f, _sz = C.c_void_p, C.c_int, C.c_long, C.c_float, C.c_size_t
_psz = C.POINTER(C.c_size_t)
_pcfg = C.POINTER(StageCfg)

_SIGS = {
    "rp_ctx_create": [C.POINTER(_vp), _i, _vp, _vp, _pcfg],
    "rp_ctx_destroy": [_vp],
    "rp_query_sizes": [_pcfg, _i, _i, _psz, _psz, _psz],
    "rp_slot_bytes": [_pcfg, _psz],
    "rp_weight_layout": [_pcfg, _i, _i, _psz, _psz],
    "rp_grad_layout": [_pcfg, _i, _i, _psz, _psz],
    "rp_weight_chunk": [_pcfg, _i, _psz, _psz],
    "rp_stage_upload_weights": [_vp, _i, _vp, _vp, _sz],
    "rp_stage_bind_weights": [_vp, _i, _vp, _sz],
    "rp_stage_forward": [_vp, _i, _vp, _vp, C.POINTER(_vp), _vp, _i, _i, _vp, _sz],
    "rp_stage_backward": [_vp, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _vp, _sz],
    "rp_lmhead_ce_fwd_bwd": [_vp, _i, _vp, _vp, _vp, _vp, _vp, _f, _i, _i, _vp, _sz],
    "rp_plan_transfers": [_psz, _i, _i, _sz, C.POINTER(Piece), _i, C.POINTER(_i)],
    "rp_partition_stages": [_i, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                            C.c_double, _i, _i, C.POINTER(_i), C.POINTER(_i), C.POINTER(_i), C.POINTER(_i),
                            C.POINTER(C.c_double), C.POINTER(C.c_double)],
    "rp_ctx_set_transfer_streams": [_vp, _vp, _vp, _vp],
    "rp_round_forward": [_vp, _i, C.POINTER(RoundIO), _i, _i, _vp, _sz],
    "rp_round_backward": [_vp, _i, C.POINTER(RoundIO), _vp, _i, _i, _vp, _sz],
    "rp_trace_start": [_vp, _i],
    "rp_trace_stop": [_vp, C.POINTER(TraceRecord), _i, C.POINTER(_i)],
    "rp_op_gemm": [_vp, _i, _i, _vp, _vp, _vp, _i, _i, _i, _l, _l, _l, _f, _i, _vp, _vp, _i, _l, _l, _vp, _l, _i, _vp, _sz],
    "rp_op_gemm_arrange": [_vp, _vp, _l, _i, _i, _i, _vp, _sz],
    "rp_op_rmsnorm_fwd": [_vp, _vp, _vp, _vp, _vp, _i, _i, _f],
    "rp_op_rmsnorm_bwd": [_vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i],
    "rp_op_rmsnorm_bwd_noalloc": [_vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i],
    "rp_op_rope_table": [_vp, _vp, _i, _i, _f],
    "rp_op_qknorm_rope": [_vp, _i, _i, _vp, _vp, _l, _l, _vp, _vp, _l, _l, _vp, _vp, _vp, _vp, _vp, _vp, _l, _vp, _vp,
                          _vp, _vp, _i, _i, _i, _i, _i, _f],
    "rp_op_swiglu_fwd": [_vp, _vp, _vp, _l, _i],
    "rp_op_swiglu_bwd": [_vp, _vp, _vp, _vp, _l, _i],
    "rp_op_moe_route_plan": [_vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "rp_op_attn_fwd": [_vp, _vp, _vp, _vp, _vp, _vp, _l, _l, _l, _l, _i, _i, _i, _i, _i],
    "rp_op_attn_bwd": [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _l, _l, _l, _l, _l, _l, _l, _l, _i, _i, _i,
                       _i, _i],
}
EXPORTS = sorted(list(_SIGS) + ["rp_last_error"])
for _name, _args in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.argtypes = _args
    _fn.restype = _i
lib.rp_last_error.argtypes = [_vp]
lib.rp_last_error.restype = C.c_char_p


def _ptr(t):
    """torch tensor / int / None -> address."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _check(code, ctx=None):
    if code != RP_OK:
        msg = lib.rp_last_error(ctx)
        raise RpError(code, msg.decode() if msg else "")


def make_cfg(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab=0, n_experts=0, top_k=0, rope_base=1.0e6,
             rms_eps=1.0e-6, qk_norm=1, lora_rank=0, lora_scale=1.0, lora=(), train_base=1, moe_router=0, head_chunk=0,
             head_two_sweeps=0):
    mask = 0
    for name in lora:
        mask |= LORA_BITS[name]
    return StageCfg(C.sizeof(StageCfg), n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, n_experts, top_k,
                    rope_base, rms_eps, int(qk_norm), lora_rank, lora_scale, mask if lora_rank > 0 else 0, int(train_base),
                    int(moe_router), int(head_chunk), int(head_two_sweeps))


# ---- rp.h ---------------------------------------------------------------------------------------------------------
def rp_query_sizes(cfg, batch, seq):
    w, g, ws = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib.rp_query_sizes(C.byref(cfg), batch, seq, C.byref(w), C.byref(g), C.byref(ws)))
    return w.value, g.value, ws.value


def rp_slot_bytes(cfg):
    n = C.c_size_t()
    _check(lib.rp_slot_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def rp_weight_layout(cfg, layer, tensor_id):
    off, n = C.c_size_t(), C.c_size_t()
    _check(lib.rp_weight_layout(C.byref(cfg), layer, tensor_id, C.byref(off), C.byref(n)))
    return off.value, n.value


def rp_grad_layout(cfg, layer, tensor_id):
    off, n = C.c_size_t(), C.c_size_t()
    _check(lib.rp_grad_layout(C.byref(cfg), layer, tensor_id, C.byref(off), C.byref(n)))
    return off.value, n.value


def rp_weight_chunk(cfg, layer):
    b, e = C.c_size_t(), C.c_size_t()
    _check(lib.rp_weight_chunk(C.byref(cfg), layer, C.byref(b), C.byref(e)))
    return b.value, e.value


def rp_ctx_create(device, compute_stream, copy_stream, cfg):
    out = C.c_void_p()
    _check(lib.rp_ctx_create(C.byref(out), device, compute_stream, copy_stream, C.byref(cfg)))
    return out.value


def rp_ctx_destroy(ctx):
    _check(lib.rp_ctx_destroy(ctx))


def rp_stage_upload_weights(ctx, slot_id, dev_slot, host_blob, nbytes):
    _check(lib.rp_stage_upload_weights(ctx, slot_id, _ptr(dev_slot), _ptr(host_blob), nbytes), ctx)


def rp_stage_bind_weights(ctx, slot_id, dev_slot, nbytes):
    _check(lib.rp_stage_bind_weights(ctx, slot_id, _ptr(dev_slot), nbytes), ctx)


def rp_stage_forward(ctx, slot_id, x_in, x_out, layer_inputs_out, router_logits, batch, seq, workspace, workspace_bytes):
    arr = None
    if layer_inputs_out is not None:
        arr = (C.c_void_p * len(layer_inputs_out))(*[_ptr(t) for t in layer_inputs_out])
    _check(lib.rp_stage_forward(ctx, slot_id, _ptr(x_in), _ptr(x_out), arr, _ptr(router_logits), batch, seq,
                                _ptr(workspace), workspace_bytes), ctx)


def rp_stage_backward(ctx, slot_id, phases, x_in, dy, dx, x_out, grads, router_logits, d_router_logits, batch, seq,
                      workspace, workspace_bytes):
    _check(lib.rp_stage_backward(ctx, slot_id, phases, _ptr(x_in), _ptr(dy), _ptr(dx), _ptr(x_out), _ptr(grads),
                                 _ptr(router_logits), _ptr(d_router_logits), batch, seq, _ptr(workspace),
                                 workspace_bytes), ctx)


def rp_lmhead_ce_fwd_bwd(ctx, slot_id, x, labels, loss_out, dx, grads, grad_scale, batch, seq, workspace,
                         workspace_bytes):
    _check(lib.rp_lmhead_ce_fwd_bwd(ctx, slot_id, _ptr(x), _ptr(labels), _ptr(loss_out), _ptr(dx), _ptr(grads),
                                    grad_scale, batch, seq, _ptr(workspace), workspace_bytes), ctx)


def rp_plan_transfers(item_bytes, n_windows, max_piece_bytes):
    """Returns the pieces as (item, window, offset, bytes) tuples in the order they were assigned."""
    n = len(item_bytes)
    arr = (C.c_size_t * max(n, 1))(*item_bytes)
    cnt = C.c_int()
    code = lib.rp_plan_transfers(arr, n, n_windows, max_piece_bytes, None, 0, C.byref(cnt))
    if code not in (RP_OK, RP_ENOMEM):
        raise RpError(code, "rp_plan_transfers: bad arguments")
    buf = (Piece * max(cnt.value, 1))()
    code = lib.rp_plan_transfers(arr, n, n_windows, max_piece_bytes, buf, cnt.value, C.byref(cnt))
    if code != RP_OK:
        raise RpError(code, "rp_plan_transfers failed")
    return [(buf[i].item, buf[i].window, buf[i].offset, buf[i].bytes) for i in range(cnt.value)]


def rp_partition_stages(t_fwd, t_bwd, mem_fwd, mem_bwd, mem_limit, n_gpus, n_micro):
    """Returns (forward stage sizes, backward stage sizes with B_1 first, t_max, cost)."""
    n = len(t_fwd)
    arr = lambda v: (C.c_double * n)(*[float(x) for x in v])
    fl, bl = (C.c_int * n)(), (C.c_int * n)()
    nf, nb, tm, cost = C.c_int(), C.c_int(), C.c_double(), C.c_double()
    code = lib.rp_partition_stages(n, arr(t_fwd), arr(t_bwd), arr(mem_fwd), arr(mem_bwd), float(mem_limit), n_gpus, n_micro,
                                   fl, C.byref(nf), bl, C.byref(nb), C.byref(tm), C.byref(cost))
    if code != RP_OK:
        raise RpError(code, "rp_partition_stages failed")
    return list(fl[:nf.value]), list(bl[:nb.value]), tm.value, cost.value


def rp_ctx_set_transfer_streams(ctx, act_up, act_down, grad_down):
    _check(lib.rp_ctx_set_transfer_streams(ctx, act_up, act_down, grad_down), ctx)


def make_round_io(x_host, out_host, x_dev, out_dev, dy_host=None, dy_dev=None, next_slot=-1, next_dev_slot=None,
                  next_host_blob=None, done_grads_dev=None, done_grads_host=None, max_piece_bytes=0):
    """Lists of torch tensors (pinned host / device) -> RoundIO.  The returned object keeps the pointer arrays alive."""
    m = len(x_host)
    io = RoundIO()
    io.struct_size = C.sizeof(RoundIO)
    io.n_micro = m
    io._keep = [(C.c_void_p * m)(*[_ptr(t) for t in x_host]), (C.c_void_p * m)(*[_ptr(t) for t in out_host]),
                (C.c_void_p * m)(*[_ptr(t) for t in dy_host]) if dy_host is not None else None]
    io.x_host = C.cast(io._keep[0], C.POINTER(C.c_void_p))
    io.out_host = C.cast(io._keep[1], C.POINTER(C.c_void_p))
    if dy_host is not None:
        io.dy_host = C.cast(io._keep[2], C.POINTER(C.c_void_p))
    for b in range(2):
        io.x_dev[b] = _ptr(x_dev[b])
        io.out_dev[b] = _ptr(out_dev[b])
        if dy_dev is not None:
            io.dy_dev[b] = _ptr(dy_dev[b])
    io.next_slot = next_slot
    io.next_dev_slot = _ptr(next_dev_slot)
    io.next_host_blob = _ptr(next_host_blob)
    io.done_grads_dev = _ptr(done_grads_dev)
    io.done_grads_host = _ptr(done_grads_host)
    io.max_piece_bytes = max_piece_bytes
    return io


def rp_round_forward(ctx, slot_id, io, batch, seq, workspace, workspace_bytes):
    _check(lib.rp_round_forward(ctx, slot_id, C.byref(io), batch, seq, _ptr(workspace), workspace_bytes), ctx)


def rp_round_backward(ctx, slot_id, io, grads, batch, seq, workspace, workspace_bytes):
    _check(lib.rp_round_backward(ctx, slot_id, C.byref(io), _ptr(grads), batch, seq, _ptr(workspace), workspace_bytes), ctx)


# ---- rp_ops.h -----------------------------------------------------------------------------------------------------
def rp_trace_start(ctx, max_records):
    _check(lib.rp_trace_start(ctx, max_records), ctx)


def rp_trace_stop(ctx, cap):
    """Returns a list of (name, flops, bytes, ms) in launch order."""
    buf = (TraceRecord * cap)()
    n = C.c_int()
    _check(lib.rp_trace_stop(ctx, buf, cap, C.byref(n)), ctx)
    return [(buf[i].name.decode(), buf[i].flops, buf[i].bytes, buf[i].ms) for i in range(n.value)]


def rp_op_gemm(stream, layout, out_f32, A, B, Cm, M, N, K, lda, ldb, ldc, alpha=1.0, beta=0, A2=None, B2=None, K2=0,
               lda2=0, ldb2=0, R=None, ldr=0, tile=0, split_ws=None):
    _check(lib.rp_op_gemm(stream, layout, out_f32, _ptr(A), _ptr(B), _ptr(Cm), M, N, K, lda, ldb, ldc, alpha, beta,
                          _ptr(A2), _ptr(B2), K2, lda2, ldb2, _ptr(R), ldr, tile, _ptr(split_ws),
                          split_ws.numel() * split_ws.element_size() if split_ws is not None else 0))


def rp_op_gemm_arrange(stream, Bm, ldb, N, K, transposed, out):
    _check(lib.rp_op_gemm_arrange(stream, _ptr(Bm), ldb, N, K, transposed, _ptr(out), out.numel() * out.element_size()))


def rp_op_rmsnorm_fwd(stream, x, g, y, rstd, T_, h, eps):
    _check(lib.rp_op_rmsnorm_fwd(stream, _ptr(x), _ptr(g), _ptr(y), _ptr(rstd), T_, h, eps))


def rp_op_rmsnorm_bwd(stream, dy, dy_is_f32, x, g, rstd, dres, dx, dg, scratch, T_, h):
    _check(lib.rp_op_rmsnorm_bwd(stream, _ptr(dy), dy_is_f32, _ptr(x), _ptr(g), _ptr(rstd), _ptr(dres), _ptr(dx),
                                 _ptr(dg), _ptr(scratch), T_, h))


def rp_op_rmsnorm_bwd_noalloc(stream, dy, dy_is_f32, x, g, rstd, dres, dx, dg, T_, h):
    _check(lib.rp_op_rmsnorm_bwd_noalloc(stream, _ptr(dy), dy_is_f32, _ptr(x), _ptr(g), _ptr(rstd), _ptr(dres), _ptr(dx),
                                         _ptr(dg), T_, h))


def rp_op_rope_table(stream, cs, seq, d, base):
    _check(lib.rp_op_rope_table(stream, _ptr(cs), seq, d, base))


def rp_op_qknorm_rope(stream, bwd, d, in_q, in_k, ld_in_q, ld_in_k, out_q, out_k, ld_out_q, ld_out_k, gq, gk, rstd_q,
                      rstd_k, raw_q, raw_k, ld_raw, dgq, dgk, scratch, cs, T_, seq, a, k, use_norm, eps):
    _check(lib.rp_op_qknorm_rope(stream, bwd, d, _ptr(in_q), _ptr(in_k), ld_in_q, ld_in_k, _ptr(out_q), _ptr(out_k),
                                 ld_out_q, ld_out_k, _ptr(gq), _ptr(gk), _ptr(rstd_q), _ptr(rstd_k), _ptr(raw_q),
                                 _ptr(raw_k), ld_raw, _ptr(dgq), _ptr(dgk), _ptr(scratch), _ptr(cs), T_, seq, a, k,
                                 use_norm, eps))


def rp_op_swiglu_fwd(stream, gu, act, T_, m):
    _check(lib.rp_op_swiglu_fwd(stream, _ptr(gu), _ptr(act), T_, m))


def rp_op_swiglu_bwd(stream, dact, gu, dgu, T_, m):
    _check(lib.rp_op_swiglu_bwd(stream, _ptr(dact), _ptr(gu), _ptr(dgu), T_, m))


def rp_op_moe_route_plan(stream, logits, T_, E, top_k, idx, w, counts, seg, tile_tab, ntiles, slot_of, row_tok, hist):
    _check(lib.rp_op_moe_route_plan(stream, _ptr(logits), T_, E, top_k, _ptr(idx), _ptr(w), _ptr(counts), _ptr(seg),
                                    _ptr(tile_tab), _ptr(ntiles), _ptr(slot_of), _ptr(row_tok), _ptr(hist)))


def rp_op_attn_fwd(stream, q, k, v, o, lse, ldq, ldk, ldv, ldo, batch, seq, a, kh, d):
    _check(lib.rp_op_attn_fwd(stream, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), ldq, ldk, ldv, ldo, batch, seq, a,
                              kh, d))


def rp_op_attn_bwd(stream, q, k, v, o, dout, lse, delta, dq, dk, dv, scratch, ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv,
                   batch, seq, a, kh, d):
    _check(lib.rp_op_attn_bwd(stream, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(dout), _ptr(lse), _ptr(delta), _ptr(dq),
                              _ptr(dk), _ptr(dv), _ptr(scratch), ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv, batch, seq, a,
                              kh, d))
