"""CPU oracle for the RoundPipe worker hot path (decoder-stage forward/backward, LM head + loss).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow numpy implementation of what one
pipeline stage computes (paper Sec. 3.2 "asymmetric stage splitting": a backward stage re-runs
the forward of its layers and then back-propagates; Sec. 4.1.1: the last stage returns a scalar
loss and gradients accumulate in place).  It exists so that the HIP library can be checked
against something that shares no code with it.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product package never does.

Every formula is the textbook definition written out (no blocking, no fusion, no re-ordering).
The layer-level math (RMSNorm, LoRA, RoPE, GQA attention, SwiGLU, top-k MoE, cross-entropy) is
not spelled out by the paper, which treats a layer as a black box; the definitions used here are
the public Qwen3-style ones and every choice where the paper is silent is listed in the
repository's design notes.

Parity status: all functions are pinned by closed forms, invariants, brute-force loops and
central finite differences (tests/test_oracle_*.py).  Full-size numeric outputs have no printed
values in the paper to compare with: for those the status is "parity unpinned by the paper".
"""
from .config import StageConfig  # noqa: F401
