"""The entry point that allocates nothing, jf_layernorm_q_bwd_static (run with -m gpu; collected last on purpose).

It must give, bit for bit, what jf_layernorm_q_bwd gives with a caller-provided workspace: on two calls in a row, the
second on a smaller input (the static scratch keeps the first call's contents), without allocating device memory."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_12422_amd as jf
from paper_2403_12422_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, N, C, block):
    x, gamma, beta, gr = workloads.layernorm_case(seed, N, C)
    (X, SX), (G, SG) = oracle.quantize_block(x, block), oracle.quantize_block(gr, block)
    _, _, mean, rstd, _ = oracle.layernorm_q(X, SX, gamma, beta, 1e-5, block)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return tuple(to(a) for a in (G, SG, X, SX, gamma, mean, rstd))


def _outputs(N, C, block):
    return (torch.empty((N, C), dtype=torch.int8, device=DEV), torch.empty((N // block, C // block), dtype=torch.float32, device=DEV),
            torch.empty((C,), dtype=torch.float32, device=DEV), torch.empty((C,), dtype=torch.float32, device=DEV))


@pytest.mark.parametrize("block,first,second", [(32, (4096, 768), (96, 352)), (64, (256, 2304), (128, 192)),
                                                (128, (1024, 1280), (256, 384)), (32, (19200, 96), (64, 4096))])
def test_static_scratch_matches_workspace_entry_point(block, first, second):
    for (N, C) in (first, second):                           # two calls in a row, the second on a smaller input
        print(f"layernorm bwd without allocation: block={block} {N}x{C}", flush=True)
        args = _case(7700 + block + N, N, C, block)
        want = jf.jf_layernorm_q_bwd(*args, block)
        out = _outputs(N, C, block)
        for t in out:
            t.fill_(-1)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        got = jf.jf_layernorm_q_bwd_static(*args, out=out, block=block)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before       # torch's allocator was not touched either
        for g, w, name in zip(got, want, ("dX", "SdX", "dgamma", "dbeta")):
            assert torch.equal(g, w), name
        # and a second time on the same input: same bits (the scratch's previous contents do not matter)
        got2 = jf.jf_layernorm_q_bwd_static(*args, out=_outputs(N, C, block), block=block)
        for g, w in zip(got2, want):
            assert torch.equal(g, w)
        del args, want, out, got, got2                       # so that the next round's allocation count starts clean


def test_static_scratch_rejects_what_does_not_fit():
    N, C, block = 16384, 4096, 64                            # 512 partial rows of 32 KiB: 16 MiB
    assert jf.jf_workspace_bytes(7, N, C, 0, block) > (8 << 20)
    args = tuple(torch.zeros(s, dtype=d, device=DEV) for s, d in (((N, C), torch.int8), ((N // block, C // block), torch.float32),
                                                                ((N, C), torch.int8), ((N // block, C // block), torch.float32),
                                                                ((C,), torch.float32), ((N,), torch.float32), ((N,), torch.float32)))
    with pytest.raises(jf.JetfireError) as err:
        jf.jf_layernorm_q_bwd_static(*args, out=_outputs(N, C, block), block=block)
    assert err.value.code == 5                               # JF_ERR_WORKSPACE
