"""The entry point that allocates nothing, signmuon_momentum_noalloc, against signmuon_momentum.

Two calls in a row through the C ABI, the second on a smaller input, each compared bit for bit with the
ordinary entry point on the same inputs (which the parity tests hold to the float32 oracle): the momentum, its
bf16 copy and the sums of squares whose partial sums live in the library's static scratch array.
"""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both(P, ctx, M, r, c, wd, stream):
    g = wl.normal((M, r, c), stream=stream, block=r, worker=c)
    m0 = wl.normal((M, r, c), stream=stream + 1, block=r, worker=c)
    w = wl.weights(r, c, stream=stream)
    out = []
    for fn in (P.signmuon_momentum, P.signmuon_momentum_noalloc):
        mom = dev(m0)
        x = torch.full((M, r, c), 7.0, dtype=torch.bfloat16, device="cuda")
        ss = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
        fn(ctx, mom, dev(g), dev(w) if wd else None, 0.9, wd, x_bf16=x, sumsq=ss)
        torch.cuda.synchronize()
        out.append((mom.cpu().numpy(), x.view(torch.int16).cpu().numpy(), ss.cpu().numpy()))
    for a, b in zip(*out):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    assert np.all(out[1][2] > 0)


def test_noalloc_momentum_matches_the_allocating_entry_point_twice():
    import paper_2605_16311_amd as P
    ctx = P.Context()
    before = ctx.workspace_bytes
    both(P, ctx, 5, 1000, 2048, 0.05, 51)      # 2000 chunks per worker, ragged last chunk
    both(P, ctx, 3, 37, 53, 0.0, 53)           # smaller: two chunks per worker, scalar path
    # only the allocating entry point grew the context's scratch; a fresh context that calls the
    # no-alloc entry point alone holds no device memory at all
    ctx2 = P.Context()
    g = dev(wl.normal((2, 64, 64), stream=55))
    mom = torch.zeros_like(g)
    ss = torch.zeros((2,), device="cuda")
    P.signmuon_momentum_noalloc(ctx2, mom, g, None, 0.9, 0.0, sumsq=ss)
    torch.cuda.synchronize()
    assert ctx2.workspace_bytes == 0 and before == 0
    # beyond the static scratch: rejected with a clear error, nothing queued
    M, r, c = 16, 4096, 16400                  # 16 * ceil(r c / 1024) * 4 bytes > 4 MiB
    big = torch.empty((1,), device="cuda")
    with pytest.raises(P.SignMuonError, match="static scratch"):
        P.binding._lib.signmuon_momentum_noalloc  # the symbol exists
        ctx2._check(P.binding._lib.signmuon_momentum_noalloc(
            ctx2._h, big.data_ptr(), big.data_ptr(), None, M, r, c, 0.9, 0.0, None, big.data_ptr()), "noalloc")
    ctx.close()
    ctx2.close()
