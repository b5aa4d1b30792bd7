"""nats_hybrid_attn_fwd_noalloc (the forward on the library's built-in scratch buffer, for callers that cannot
allocate) against nats_hybrid_attn_fwd with a caller workspace: same kernels, so the same bits; two calls in a row,
the second on a smaller problem, then the size limit."""
import pytest
import torch

import paper_2602_03681_amd as nats
from paper_2602_03681_amd import binding as nb
from nats_inputs import make_fwd_inputs

from gpu_util import TOL, host, oracle_fwd, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _pair(B, H, L, d, dtype, seed, **kw):
    x = make_fwd_inputs(B, H, L, d, dtype, 0.1, seed=seed)
    g = to_dev(x, dtype)
    ref = nats.hybrid_attn_fwd(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], 64, **kw)
    out = torch.full_like(g["Q"], float("nan"))
    nats.hybrid_attn_fwd_noalloc(g["Q"], g["K"], g["V"], g["alpha"], g["beta"], g["mask"], out, 64, **kw)
    torch.cuda.synchronize()
    return x, ref, out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_noalloc_forward_matches_the_workspace_forward_twice(dtype):
    view = torch.int16 if dtype == "bf16" else torch.int32
    x1, ref1, out1 = _pair(1, 3, 1024, 128, dtype, seed=901)
    assert torch.equal(out1.view(view), ref1.view(view))
    # a smaller problem through the same buffer, which still holds the first call's intermediates
    x2, ref2, out2 = _pair(2, 2, 320, 64, dtype, seed=902, combine_mode=1)
    assert torch.equal(out2.view(view), ref2.view(view))
    stored = "bf16" if dtype == "bf16" else None
    assert rel_err(host(out1), oracle_fwd(x1, want=())["O"], stored) <= TOL[dtype]
    assert rel_err(host(out2), oracle_fwd(x2, want=(), mode=1)["O"], stored) <= TOL[dtype]


def test_noalloc_forward_rejects_what_does_not_fit():
    B, H, L, d = 2, 16, 8192, 128
    p = nb.make_fwd_params(B, H, L, d, 64, nb.NATS_BF16)
    assert nb.fwd_workspace_bytes(p) > nb.NOALLOC_SCRATCH_BYTES
    q = torch.zeros((B, H, L, d), dtype=torch.bfloat16, device="cuda")
    a = torch.ones((B, H, L), dtype=torch.float32, device="cuda")
    m = torch.zeros((B, H, L), dtype=torch.uint8, device="cuda")
    with pytest.raises(nb.NatsError, match="scratch"):
        nats.hybrid_attn_fwd_noalloc(q, q, q, a, a, m, torch.empty_like(q), 64)
