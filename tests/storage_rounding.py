"""What bf16 STORAGE alone costs: the oracle's own layer functions with their results rounded to bf16 wherever a 16-bit
implementation has to keep a tensor in memory between two kernels (matrix-core operands and the activations that feed
them).  Nothing else changes -- same definitions, same order, same working precision inside every function -- so the
distance between this run and the plain oracle is the error floor that the storage format sets for a given workload,
independent of any kernel.  Test infrastructure: it wraps functions of oracle.layers for the duration of a `with`
block and shares nothing with the HIP path.

Rounded: RMSNorm output over the hidden axis (n1, n2), every projection output (q, k, v, gate, up, and the o / down
outputs before they join the residual stream), rotated q and k, the attention output, the SwiGLU output; in the
backward every activation gradient a projection, the SwiGLU, the attention or a norm hands on.  Not rounded (fp32 on
the device as well): norm statistics, softmax statistics, weight gradients, the loss.  The probabilities inside the
attention and the head's internals are left exact, so the floor reported here is slightly below that of a real
16-bit pipeline."""
import contextlib

import numpy as np

import synth
from oracle import layers as L


def _r(v):
    return synth.bf16_round(np.asarray(v, dtype=np.float32)).astype(v.dtype)


@contextlib.contextmanager
def bf16_storage():
    names = ["rmsnorm_fwd", "rmsnorm_bwd", "linear_fwd", "linear_bwd", "rope_fwd", "attention_fwd", "attention_bwd",
             "swiglu_fwd", "swiglu_bwd"]
    orig = {n: getattr(L, n) for n in names}

    def rmsnorm_fwd(x, g, eps):
        y, rstd = orig["rmsnorm_fwd"](x, g, eps)
        return (_r(y) if x.ndim == 2 else y), rstd          # per-head q/k norm: the rounding follows the rotation

    def rmsnorm_bwd(dy, x, g, rstd):
        dx, dg = orig["rmsnorm_bwd"](dy, x, g, rstd)
        return _r(dx), dg

    def linear_fwd(u, W, lora=None, scale=1.0):
        return _r(orig["linear_fwd"](u, W, lora, scale))

    def linear_bwd(dy, u, W, lora=None, scale=1.0, want_dW=True):
        du, dW, dA, dB = orig["linear_bwd"](dy, u, W, lora, scale, want_dW)
        return _r(du), dW, dA, dB

    def rope_fwd(u, batch, seq, base):
        return _r(orig["rope_fwd"](u, batch, seq, base))

    def attention_fwd(q, k, v, batch, seq):
        o, P, lse = orig["attention_fwd"](q, k, v, batch, seq)
        return _r(o), P, lse

    def attention_bwd(do, q, k, v, o, P_all, batch, seq):
        dq, dk, dv = orig["attention_bwd"](do, q, k, v, o, P_all, batch, seq)
        return _r(dq), _r(dk), _r(dv)

    def swiglu_fwd(gate, up):
        return _r(orig["swiglu_fwd"](gate, up))

    def swiglu_bwd(dact, gate, up):
        dg, du = orig["swiglu_bwd"](dact, gate, up)
        return _r(dg), _r(du)

    new = dict(rmsnorm_fwd=rmsnorm_fwd, rmsnorm_bwd=rmsnorm_bwd, linear_fwd=linear_fwd, linear_bwd=linear_bwd,
               rope_fwd=rope_fwd, attention_fwd=attention_fwd, attention_bwd=attention_bwd, swiglu_fwd=swiglu_fwd,
               swiglu_bwd=swiglu_bwd)
    try:
        for n, f in new.items():
            setattr(L, n, f)
        yield
    finally:
        for n, f in orig.items():
            setattr(L, n, f)
