"""curdkv_adaptive_budgets_noalloc, the entry point for callers that cannot allocate
device memory: its budgets must equal, bit for bit, those of curdkv_adaptive_budgets
(which allocates its workspace on first use) on the same scores, also on a second
call with a smaller input right after the first (the static workspace keeps the first
call's contents), and sizes beyond its fixed workspace must be refused before
anything is launched.  Called through the C ABI."""

import sys

import numpy as np
import pytest

from oracle import curdkv_oracle as orc
from paper_2509_15038_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


def _scores(heads, n, seed):
    rng = np.random.default_rng(seed)
    sc = (rng.random((heads, n)) ** 6).astype(np.float32)
    sc[:, : n // 2] = np.round(sc[:, : n // 2] * 256) / 256    # planted ties inside a head ...
    if heads > 1:
        sc[1] = sc[0]                                          # ... and across two heads of a layer
    sc /= sc.sum(1, keepdims=True)
    return sc


def test_noalloc_budgets_equal_the_allocating_entry_point():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    B.lib()
    L, H = 6, 8
    heads = L * H
    n_big, n_small = 20000 + 13, 3000 + 5
    with B.Context(L, H, 4, 128, 64, "bf16", n_big, 1) as ctx:
        # two calls in a row on the same context, the second on a smaller input
        for call, (n, k, s, alpha) in enumerate([(n_big, n_big // 10, 4, 0.2), (n_small, n_small // 5, 4, 0.2),
                                                 (n_small, n_small // 3, 0, 0.0), (n_big, n_big // 20, 64, 0.5)]):
            sc = _scores(heads, n, 100 + call)
            sc_d = torch.from_numpy(sc).cuda()
            want = torch.full((heads,), -7, dtype=torch.int32, device="cuda")
            got = torch.full((heads,), -9, dtype=torch.int32, device="cuda")
            ctx.adaptive_budgets_noalloc(sc_d, n, k, s, alpha, got)
            ctx.adaptive_budgets(sc_d, n, k, s, alpha, want)
            torch.cuda.synchronize()
            assert torch.equal(got, want), (call, n, k, s, alpha)
            # and both are the oracle's allocation on these very scores (fp32 values are exact in float64)
            got_h = got.cpu().numpy()
            for l in range(L):
                ref = orc.adaptive_budgets(sc[l * H:(l + 1) * H].astype(np.float64), k, s, alpha)
                assert got_h[l * H:(l + 1) * H].tolist() == ref.tolist(), (call, l)
    # a smaller context afterwards: fewer heads, fewer layers, the same static workspace
    with B.Context(1, 3, 4, 128, 32, "fp32", 900, 2) as ctx:
        sc = _scores(3, 900, 7)
        sc_d = torch.from_numpy(sc).cuda()
        want = torch.empty((3,), dtype=torch.int32, device="cuda")
        got = torch.empty((3,), dtype=torch.int32, device="cuda")
        ctx.adaptive_budgets_noalloc(sc_d, 900, 100, 4, 0.2, got)
        ctx.adaptive_budgets(sc_d, 900, 100, 4, 0.2, want)
        # nothing to allot (budget inside the sinks; safeguard covering every place): no workspace use at all
        for (k, s, alpha) in [(3, 4, 0.2), (50, 4, 1.0), (0, 4, 0.2)]:
            a = torch.empty((3,), dtype=torch.int32, device="cuda")
            b = torch.empty((3,), dtype=torch.int32, device="cuda")
            ctx.adaptive_budgets_noalloc(sc_d, 900, k, s, alpha, a)
            ctx.adaptive_budgets(sc_d, 900, k, s, alpha, b)
            torch.cuda.synchronize()
            assert torch.equal(a, b) and int(a.sum()) == 3 * k
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        assert got.cpu().numpy().tolist() == orc.adaptive_budgets(sc.astype(np.float64), 100, 4, 0.2).tolist()


def test_noalloc_rejects_what_its_workspace_cannot_hold():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    # 1025 (layer, group) pairs: one more than the static workspace is sized for
    with B.Context(1025, 1, 1, 128, 32, "bf16", 64, 3) as ctx:
        sc = torch.full((1025, 64), 1.0 / 64, dtype=torch.float32, device="cuda")
        out = torch.full((1025,), -7, dtype=torch.int32, device="cuda")
        with pytest.raises(B.CurdkvError) as e:
            ctx.adaptive_budgets_noalloc(sc, 64, 10, 4, 0.2, out)
        assert e.value.code == B.ERR_TOO_LARGE and "workspace" in B.strerror(B.ERR_TOO_LARGE)
        torch.cuda.synchronize()
        assert bool((out == -7).all())                       # nothing was launched
        ctx.adaptive_budgets(sc, 64, 10, 4, 0.2, out)         # the allocating entry point still serves this size
        torch.cuda.synchronize()
        assert bool((out == 10).all())                       # one head per layer: it keeps the layer's whole budget
    with B.Context(1024, 1, 1, 128, 32, "bf16", 64, 3) as ctx:  # exactly the limit is accepted
        sc = torch.full((1024, 64), 1.0 / 64, dtype=torch.float32, device="cuda")
        out = torch.full((1024,), -7, dtype=torch.int32, device="cuda")
        ctx.adaptive_budgets_noalloc(sc, 64, 10, 4, 0.2, out)
        torch.cuda.synchronize()
        assert bool((out == 10).all())
        # the same argument checks as the allocating entry point, before anything is launched
        for args in [(sc, 64, 65, 4, 0.2, out), (sc, 64, 10, 4, 1.5, out), (None, 64, 10, 4, 0.2, out),
                     (sc, 64, 10, 4, 0.2, None), (sc, 65, 10, 4, 0.2, out), (sc, 64, 10, -1, 0.2, out)]:
            with pytest.raises(B.CurdkvError) as e:
                ctx.adaptive_budgets_noalloc(*args)
            assert e.value.code == B.ERR_INVALID_ARG
