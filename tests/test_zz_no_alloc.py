"""The entry point that allocates nothing (rp_op_rmsnorm_bwd_noalloc: the gain-gradient partials go through an array
inside the library instead of a caller-owned scratch buffer) against the existing entry point, through the C ABI: two
calls in a row, the second with a smaller input, so that whatever the first call left in the shared array is there
when the second runs.  Both entry points run the same deterministic kernels: the results must be identical."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_rmsnorm_bwd_noalloc_matches_the_scratch_argument_version():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_27085_amd import binding as B, harness as H
    st = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(4242)
    for T, h, f32 in ((2600, 4096, 0), (333, 1024, 1)):      # more rows than partial blocks first, then a smaller input
        print("noalloc case T=%d h=%d dy_is_f32=%d" % (T, h, f32), flush=True)
        rnd = lambda shape: synth.bf16_round(rng.standard_normal(shape, dtype=np.float32))
        x, dy, dres = rnd((T, h)), rnd((T, h)), rnd((T, h))
        g = synth.bf16_round(1 + 0.1 * rng.standard_normal(h).astype(np.float32))
        xd, gd, dresd = H.bf16_tensor(x, "cuda:0"), H.bf16_tensor(g, "cuda:0"), H.bf16_tensor(dres, "cuda:0")
        dyd = torch.from_numpy(dy).cuda() if f32 else H.bf16_tensor(dy, "cuda:0")
        y = torch.empty((T, h), dtype=torch.bfloat16, device="cuda:0")
        rstd = torch.empty(T, dtype=torch.float32, device="cuda:0")
        B.rp_op_rmsnorm_fwd(st, xd, gd, y, rstd, T, h, 1e-6)
        dg0 = torch.from_numpy(rng.standard_normal(h).astype(np.float32)).cuda()      # gradients accumulate into dg
        dx_a, dx_b = torch.empty_like(y), torch.empty_like(y)
        dg_a, dg_b = dg0.clone(), dg0.clone()
        scratch = torch.empty(1024 * h, dtype=torch.float32, device="cuda:0")
        B.rp_op_rmsnorm_bwd(st, dyd, f32, xd, gd, rstd, dresd, dx_a, dg_a, scratch, T, h)
        B.rp_op_rmsnorm_bwd_noalloc(st, dyd, f32, xd, gd, rstd, dresd, dx_b, dg_b, T, h)
        torch.cuda.synchronize()
        assert torch.equal(dx_a, dx_b)
        assert torch.equal(dg_a, dg_b)
        assert not torch.equal(dg_a, dg0)
    # beyond the built-in scratch: a clear error, nothing enqueued
    with pytest.raises(B.RpError) as e:
        B.rp_op_rmsnorm_bwd_noalloc(st, dyd, f32, xd, gd, rstd, dresd, dx_b, dg_b, 8, 8192)
    assert e.value.code == B.RP_EINVAL and "4096" in str(e.value)
