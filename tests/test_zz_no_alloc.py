"""ckks_rescale_noalloc (the rescale for callers that cannot allocate: scratch in a buffer that is part of the library's
image) against ckks_rescale with a caller's workspace, through the C boundary: same residues, on two calls in a row, the
second with a smaller input (lower level), and against the oracle; sizes beyond the built-in buffer are rejected."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2604_16834_amd as hx  # noqa: E402
from oracle import Oracle  # noqa: E402
from workloads import CONFIGS, make_params  # noqa: E402
from gpu_common import rand_ct  # noqa: E402


def test_rescale_without_allocation_matches_rescale_with_workspace():
    p = CONFIGS["cfg3_rotations"].params()                 # N = 2^16, 24 limbs: the benchmark's ring
    orc, ctx = Oracle(p), hx.Context(p)
    rng = np.random.default_rng(4242)
    first = True
    for level in (p.num_q - 1, 5):                         # two calls in a row, the second smaller
        ct = rand_ct(rng, p.moduli, level, orc.N)
        d_ct = hx.from_host(ct)
        want = hx.ckks_rescale(ctx, d_ct, level)
        out = hx.empty(2, level, orc.N)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        hx.ckks_rescale_noalloc(ctx, d_ct, level, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"level {level}"
        if first:                                          # and against the oracle, once
            assert np.array_equal(hx.to_host(out), orc.rescale(ct, level))
            first = False


def test_rescale_without_allocation_small_ring_and_other_context():
    """A second context (N = 2^13, integer kernels' ring sizes included) shares the same buffer on the same GPU."""
    for log_n, num_q, bits in ((13, 7, 50), (10, 3, 57)):
        p = make_params(log_n, num_q, 1, 1, bits=bits)
        orc, ctx = Oracle(p), hx.Context(p)
        rng = np.random.default_rng(77 + log_n)
        for level in (num_q - 1, 1):
            ct = rand_ct(rng, p.moduli, level, orc.N)
            out = hx.empty(2, level, orc.N)
            hx.ckks_rescale_noalloc(ctx, hx.from_host(ct), level, out)
            assert np.array_equal(hx.to_host(out), orc.rescale(ct, level)), (log_n, level)


def test_rescale_without_allocation_rejects_what_does_not_fit():
    p = make_params(17, 20, 0, 0)                          # N = 2^17: (level + 1) * 2 MiB of scratch
    ctx = hx.Context(p)
    N = 1 << 17
    level = 19
    assert hx.ckks_workspace_bytes(ctx, hx.binding.CKKS_OP_RESCALE, level) > (32 << 20)
    ct, out = hx.empty(2, level + 1, N), hx.empty(2, level, N)
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_rescale_noalloc(ctx, ct, level, out)
    assert e.value.code == hx.binding.CKKS_ERR_UNSUPPORTED_PARAMS and "scratch" in str(e.value)
    with pytest.raises(hx.CkksError) as e:                 # level 0 has nothing to drop, as for ckks_rescale
        hx.ckks_rescale_noalloc(ctx, hx.empty(2, 1, N), 0, hx.empty(2, 1, N))
    assert e.value.code == hx.binding.CKKS_ERR_LEVEL_MISMATCH
    level = 15                                             # the largest that fits at this ring size
    ct15 = hx.from_host(rand_ct(np.random.default_rng(5), p.moduli, level, N))
    out15 = hx.empty(2, level, N)
    hx.ckks_rescale_noalloc(ctx, ct15, level, out15)
    assert torch.equal(out15, hx.ckks_rescale(ctx, ct15, level))
