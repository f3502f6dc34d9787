"""GPU parity of the kernel that keeps the scores of a strip resident across compute units (one sweep over
the keys; the workgroups that share a row exchange their row statistics through tables parked in P)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_13885_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    gu.require_gpu()


@pytest.fixture(autouse=True)
def _force(monkeypatch):
    monkeypatch.setenv("ATTNW_FUSED_KERNEL", "gang")


def _check_all(x, P, what):
    got = gu.to_f64(P)
    for b in range(x.B):
        for h in range(x.H):
            ref = oracle.attention_weights(x.Q[b, h], x.K[b, h], "bf16", x.scale)
            gu.check_weights(got[b, h], ref, "bf16", f"{what} head ({b},{h})")


# gangs of 2, 3, 5, 7, 8, 12, 14, 16 workgroups of four waves (key ranges of 256, N <= 4096) and of 10, 16 and 32 workgroups of
# eight waves (key ranges of 512, beyond 4096 keys); lists of one strip (fewer strips than gangs), lists that cross
# heads, lists of a whole head; both head sizes; sharp and flat rows; a negative scale
@pytest.mark.parametrize("B,H,N,d,scale", [(1, 1, 512, 64, None), (1, 3, 768, 128, None), (3, 3, 1024, 64, -0.2),
                                           (1, 2, 1280, 128, None), (1, 5, 2048, 128, None), (2, 3, 2048, 64, None),
                                           (1, 1, 4096, 128, None), (1, 3, 4096, 64, -0.11), (1, 40, 1024, 128, None),
                                           (1, 2, 5120, 64, None), (1, 1, 8192, 64, None), (1, 1, 16384, 64, None),
                                           (1, 1, 4608, 128, None), (1, 2, 8192, 128, -0.09), (1, 3, 3584, 128, 0.05),
                                           (1, 5, 1792, 64, None), (1, 2, 3072, 128, None)])
def test_gang_kernel_against_the_oracle(B, H, N, d, scale):
    x = wl.fused_inputs("t", "bf16", B, H, N, d, seed=7100 + H + N + d, scale=scale, row_factor=(0.5, 3.0))
    P = gu.run_fused(x, guard=8192)
    _check_all(x, P, f"gang kernel {B}x{H}x{N}x{d}")


def test_gang_kernel_is_deterministic_and_ignores_what_p_held():
    """The exchange tables are parked in P: whatever P held before the call (all ones, NaN patterns, the
    previous result) must not matter, and two calls give the same bits."""
    x = wl.fused_inputs("t", "bf16", 1, 4, 2048, 128, seed=7200, row_factor=(0.5, 3.0))
    import paper_2407_13885_amd as attnw
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    outs = []
    for fill in (0x3f80, 0xffff, 0x7fc0, None):
        P = torch.empty((x.B, x.H, x.N, x.N), dtype=torch.bfloat16, device="cuda")
        if fill is None:
            P.copy_(outs[0])
        else:
            P.view(torch.int16).fill_(fill - 0x10000 if fill >= 0x8000 else fill)
        attnw.attnw_fused(Q, K, P, x.B, x.H, x.N, x.d, float(x.scale), attnw.ATTNW_BF16)
        torch.cuda.synchronize()
        outs.append(P)
    for o in outs[1:]:
        assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16))
    _check_all(x, outs[0], "gang kernel, prefilled P")


def test_gang_members_that_run_at_different_speeds():
    """Gangs of 14 workgroups put 448 workgroups on a chip that holds 512: some share a compute unit and some do
    not, so the members of a gang drift apart and the fast ones wait for the slow ones' tables.  A member that has
    just published a table must still find its peers' tables of the strip before (the parking place of a table is
    not rewritten until every peer has folded it): repeated calls, over whatever P held, give the bits of the first,
    which is checked against the oracle."""
    import paper_2407_13885_amd as attnw
    x = wl.fused_inputs("t", "bf16", 1, 3, 3584, 128, seed=7300, scale=0.05, row_factor=(0.5, 2.5))
    Q, K = gu.to_dev(x.Q, "bf16"), gu.to_dev(x.K, "bf16")
    first = None
    for rep in range(12):
        P = torch.empty((x.B, x.H, x.N, x.N), dtype=torch.bfloat16, device="cuda")
        if rep % 3 == 1:
            P.view(torch.int16).fill_(0x3f80)
        if rep % 3 == 2:
            P.view(torch.int16).fill_(-1)
        attnw.attnw_fused(Q, K, P, x.B, x.H, x.N, x.d, float(x.scale), attnw.ATTNW_BF16)
        torch.cuda.synchronize()
        if first is None:
            first = P
            _check_all(x, first, "gang kernel, gangs of 14")
        else:
            assert torch.equal(P.view(torch.int16), first.view(torch.int16)), f"call {rep} differs from the first"
