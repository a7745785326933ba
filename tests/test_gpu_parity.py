"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Scores within 1e-3 relative (fp32 accumulation of exact
bf16 products against float64); index sets identical except for tokens whose
oracle score is within that tolerance of the cut; gathered rows bit-exact."""

import sys

import numpy as np
import pytest

from oracle import curdkv_oracle as orc
from paper_2509_15038_amd import binding as B
from paper_2509_15038_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    sys.stdout.flush()
    yield


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()                       # fail loudly if the HIP library is not built
    from tests import gpu_util
    return gpu_util


# ---- the benchmark configurations at sizes the oracle finishes in seconds ----

def test_c1_fp32_single_head(gu):
    cfg = wl.CONFIGS["c1"]
    worst, nd = gu.run_and_check(cfg, wl.budgets_for(cfg))
    print(f"c1 worst rel {worst:.2e}, near-cut differences {nd}")


def test_c2_llama_layer(gu):
    cfg = wl.CONFIGS["c2"]
    worst, nd = gu.run_and_check(cfg, wl.budgets_for(cfg))
    print(f"c2 worst rel {worst:.2e}, near-cut differences {nd}")


@pytest.mark.parametrize("keep", [0.10, 0.20, 0.50])
def test_c3_shape_reduced_ragged(gu, keep):
    # several tiles per wave, a ragged last tile, more than one layer
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=3, n=5000 + 17)
    gu.run_and_check(cfg, wl.budgets_for(cfg, keep))


def test_c4_shape_reduced_prefix_block(gu):
    cfg = wl.scaled(wl.CONFIGS["c4"], layers=2, n=4096 + 5)
    gu.run_and_check(cfg, wl.budgets_for(cfg), n_sink=4)
    gu.run_and_check(cfg, wl.budgets_for(cfg), n_sink=64)
    gu.run_and_check(cfg, wl.budgets_for(cfg), n_sink=0)


def test_c5_shape_reduced_dirichlet_r128_streaming_select(gu):
    # n above what LDS holds -> the select kernel streams keys from memory
    cfg = wl.scaled(wl.CONFIGS["c5"], layers=2, kv_heads=4, n=45000 + 3)
    b = wl.budgets_for(cfg)
    assert b.reshape(2, 4).sum(1).tolist() == [int(0.05 * 4 * cfg.n)] * 2
    gu.run_and_check(cfg, b)


# ---- sketch widths (the paper's r = 20 is zero-padded to 32 columns).  Below r = 8 a
# row's score can be a near-cancelled dot product, where no relative bound holds. ---

@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("r", [8, 20, 32, 48, 64, 100, 128])
def test_sketch_dims(gu, dtype, r):
    cfg = wl.scaled(wl.CONFIGS["c2"], kv_heads=2, n=700, r=r, dtype=dtype)
    gu.run_and_check(cfg, wl.budgets_for(cfg))


# ---- sizes around tile boundaries and degenerate budgets ----------------------

@pytest.mark.parametrize("n", [1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 1023, 1025])
def test_small_and_ragged_n(gu, n):
    cfg = wl.scaled(wl.CONFIGS["c2"], kv_heads=3, n=n)
    k = max(0, n // 3)
    gu.run_and_check(cfg, np.full(3, k, dtype=np.int32))


def test_degenerate_budgets(gu):
    cfg = wl.scaled(wl.CONFIGS["c2"], layers=2, kv_heads=4, n=300)
    n = cfg.n
    # empty head, inside the sinks, exactly the sinks, one above, all but one, all
    b = np.array([0, 3, 4, 5, n - 1, n, 1, 150], dtype=np.int32)
    gu.run_and_check(cfg, b, n_sink=4)
    gu.run_and_check(cfg, b, n_sink=0)
    gu.run_and_check(cfg, b, n_sink=n + 5)          # more sinks than tokens
    gu.run_and_check(cfg, np.zeros(8, dtype=np.int32))  # nothing kept anywhere


def test_zero_cache_gives_uniform_scores(gu):
    import torch
    cfg = wl.scaled(wl.CONFIGS["c2"], kv_heads=2, n=200)
    K = np.zeros((1, 2, 200, 128), dtype=np.uint16)
    _, V = wl.host_cache(cfg)
    gu.run_and_check(cfg, np.array([50, 7], dtype=np.int32), K=K, V=V)


def test_select_ties_lowest_index_first(gu):
    # planted equal scores: the choice among equals is by token index
    import torch
    n, H, s = 3000, 4, 4
    rng = np.random.default_rng(11)
    sc = rng.integers(1, 6, size=(H, n)).astype(np.float32) / 8.0
    sc[1] = 0.25                                    # one head entirely tied
    sc[2, 100:] = 0.0                               # zeros beyond a few
    budgets = np.array([700, 1234, 500, 2999], dtype=np.int32)
    off = wl.offsets_for(budgets)
    with B.Context(1, H, 4, 128, 64, "bf16", n, 1) as ctx:
        scd = torch.from_numpy(sc).cuda()
        idx = torch.full((int(off[-1]),), -1, dtype=torch.int32, device="cuda")
        ctx.select(scd, n, budgets, s, off, idx)
        torch.cuda.synchronize()
        idx = idx.cpu().numpy()
    for h in range(H):
        want = orc.select(sc[h].astype(np.float64), int(budgets[h]), s)
        assert np.array_equal(idx[off[h]:off[h + 1]], want), h


@pytest.mark.parametrize("n", [70001, 131072, 300007])
def test_select_large_n_streaming_ties(gu, n):
    # the largest n spans three of the streaming kernel's compaction blocks, with tied keys
    # on both sides of each boundary
    import torch
    H, s = 2, 4
    rng = np.random.default_rng(12)
    sc = (rng.integers(0, 50, size=(H, n)).astype(np.float32)) * np.float32(1e-6)
    budgets = np.array([n // 10, n // 2], dtype=np.int32)
    off = wl.offsets_for(budgets)
    with B.Context(1, H, 4, 128, 64, "bf16", n, 1) as ctx:
        scd = torch.from_numpy(sc).cuda()
        idx = torch.full((int(off[-1]),), -1, dtype=torch.int32, device="cuda")
        ctx.select(scd, n, budgets, s, off, idx)
        torch.cuda.synchronize()
        idx = idx.cpu().numpy()
    for h in range(H):
        want = orc.select(sc[h].astype(np.float64), int(budgets[h]), s)
        assert np.array_equal(idx[off[h]:off[h + 1]], want), h


# ---- the one-call entry point; with 256 heads (one per CU) it runs the fused kernel ----

@pytest.mark.parametrize("keep", [0.10, 0.50])
def test_one_call_fused_c3_shape(gu, keep):
    cfg = wl.scaled(wl.CONFIGS["c3"], n=2000 + 17)                   # 256 heads, ragged n
    gu.run_and_check(cfg, wl.budgets_for(cfg, keep), one_call=True, fused=True)


def test_one_call_fused_long_heads(gu):
    cfg = wl.scaled(wl.CONFIGS["c4"], n=16384 + 2048 + 33)           # second key-count variant
    gu.run_and_check(cfg, wl.budgets_for(cfg), one_call=True, fused=True)


@pytest.mark.parametrize("n", [2048, 2040, 2560, 2464, 5120 + 31, 9 * 1024])
def test_walk_start_rotation_range_lengths(gu, n):
    # A wave walks its tile range from a start that depends on head and wave, when the range is
    # whole pairs of whole tiles and at least 8 tiles long.  The sizes give the fused kernel's
    # eight waves ranges of exactly 8 tiles (2048), 8 with a ragged last tile (2040: the last
    # wave must not rotate), 10 (2560), 10 with an odd-length last range (2464 = 77 tiles), 22
    # with a ragged end, and 36; the general kernel's 4 to 32 waves per head get other lengths
    # from the same sizes.  Every score of every head is compared with the oracle, so a tile
    # walked twice or left out shows.
    cfg = wl.scaled(wl.CONFIGS["c3"], n=n)
    gu.run_and_check(cfg, wl.budgets_for(cfg, 0.1), one_call=True, fused=True)
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=2, n=n)
    gu.run_and_check(cfg, wl.budgets_for(cfg, 0.1), one_call=False)
    cfg = wl.scaled(wl.CONFIGS["c5"], layers=1, kv_heads=3, n=n)            # 128-column sketch
    gu.run_and_check(cfg, wl.budgets_for(cfg, 0.1), one_call=False)


@pytest.mark.parametrize("r", [20, 32, 64])
def test_one_call_fused_sketch_dims(gu, r):
    cfg = wl.scaled(wl.CONFIGS["c3"], n=700, r=r)
    gu.run_and_check(cfg, wl.budgets_for(cfg, 0.2), one_call=True, fused=True)


def test_one_call_fused_degenerate_budgets_and_sinks(gu):
    cfg = wl.scaled(wl.CONFIGS["c3"], n=300)
    n = cfg.n
    rng = np.random.default_rng(21)
    b = rng.choice(np.array([0, 1, 3, 4, 5, 77, n - 1, n], dtype=np.int32), size=256)
    for s in (4, 0, 64, n + 5):
        gu.run_and_check(cfg, b, n_sink=s, one_call=True, fused=True)
    gu.run_and_check(cfg, np.zeros(256, dtype=np.int32), one_call=True, fused=True)


def test_one_call_fused_zero_cache_and_ties(gu):
    cfg = wl.scaled(wl.CONFIGS["c3"], n=500)
    K, V = wl.host_cache(cfg)
    K[3] = 0                                         # a whole layer of zero keys: uniform scores, all tied
    V[5, 2, 100:] = V[5, 2, 100]                     # many identical value rows
    K[5, 2, 100:] = K[5, 2, 100]
    gu.run_and_check(cfg, wl.budgets_for(cfg, 0.3), K=K, V=V, one_call=True, fused=True)


def test_one_call_without_scores_and_fallback_paths(gu):
    import torch
    # few heads, heads that would leave the second round of CUs mostly empty, n above the LDS
    # limit, fp32: the three kernels
    for cfg in (wl.scaled(wl.CONFIGS["c2"], kv_heads=4, n=900),
                wl.scaled(wl.CONFIGS["c3"], layers=16, n=400),
                wl.scaled(wl.CONFIGS["c3"], layers=36, n=200),
                wl.scaled(wl.CONFIGS["c5"], layers=1, kv_heads=2, n=40000),
                wl.CONFIGS["c1"]):
        gu.run_and_check(cfg, wl.budgets_for(cfg), one_call=True, fused=False)
    # scores = NULL on both paths: indices and rows must equal the run that returned scores
    for cfg in (wl.scaled(wl.CONFIGS["c3"], n=1000), wl.scaled(wl.CONFIGS["c2"], kv_heads=4, n=1000),
                wl.scaled(wl.CONFIGS["c5"], layers=1, kv_heads=2, n=40000, dirichlet_total_frac=None)):
        K, V = wl.host_cache(cfg)
        Kd, Vd = gu.to_device(K, "bf16"), gu.to_device(V, "bf16")
        b = wl.budgets_for(cfg, 0.2); off = wl.offsets_for(b); tot = int(off[-1])
        with B.Context(cfg.layers, cfg.kv_heads, 4, 128, cfg.r, "bf16", cfg.n, cfg.sketch_seed) as ctx:
            _, idx, Ko, Vo, _ = gu.run_path(ctx, Kd, Vd, cfg.n, b, 4, "bf16", one_call=True)
            idx2 = torch.full((tot,), -1, dtype=torch.int32, device="cuda")
            Ko2 = torch.zeros((tot, 128), dtype=torch.bfloat16, device="cuda"); Vo2 = torch.zeros_like(Ko2)
            ctx.compress(Kd, Vd, cfg.n, b, 4, off, None, idx2, Ko2, Vo2)
            torch.cuda.synchronize()
            assert torch.equal(idx, idx2) and torch.equal(Ko.view(torch.int16), Ko2.view(torch.int16))
            assert torch.equal(Vo.view(torch.int16), Vo2.view(torch.int16))


# ---- ablation variants (appendix, "Ablation Study"): one tensor only, no projection ----

@pytest.mark.parametrize("projection", [True, False])
@pytest.mark.parametrize("source", ["kv", "k", "v"])
def test_ablation_variants(gu, source, projection):
    if source == "kv" and projection:
        pytest.skip("the method itself: covered everywhere else")
    small = wl.scaled(wl.CONFIGS["c2"], kv_heads=3, n=1500 + 7)               # three kernels
    gu.run_and_check(small, wl.budgets_for(small), source=source, projection=projection)
    gu.run_and_check(small, wl.budgets_for(small), source=source, projection=projection, one_call=True)
    fused = wl.scaled(wl.CONFIGS["c3"], n=900 + 5)                            # fused kernel
    gu.run_and_check(fused, wl.budgets_for(fused, 0.2), source=source, projection=projection, one_call=True,
                     fused=True)
    if projection:
        wide = wl.scaled(wl.CONFIGS["c5"], layers=1, kv_heads=2, n=2000, dirichlet_total_frac=None)   # r = 128
        gu.run_and_check(wide, wl.budgets_for(wide, 0.1), source=source)
    f32 = wl.CONFIGS["c1"]
    gu.run_and_check(f32, wl.budgets_for(f32), source=source, projection=projection)
    f32 = wl.scaled(wl.CONFIGS["c2"], kv_heads=3, n=2600 + 9, dtype="fp32", r=128)     # sketch in LDS; several tiles per wave
    gu.run_and_check(f32, wl.budgets_for(f32), source=source, projection=projection)


def test_ablation_config_errors(gu):
    with pytest.raises(B.CurdkvError) as e:
        B.Context(1, 1, 1, 128, 32, "bf16", 64, 1, 5, True)
    assert e.value.code == B.ERR_INVALID_ARG


# ---- AdaCurDKV head-wise budgets -----------------------------------------------------

def _ada_case(gu, scores, k, s, alpha):
    """scores: float32 [L, H, n] on the host.  GPU budgets against the oracle, layer by layer."""
    import torch
    L, H, n = scores.shape
    with B.Context(L, H, 4, 128, 64, "bf16", n, 1) as ctx:
        d = torch.from_numpy(scores).cuda()
        out = torch.full((L * H,), -1, dtype=torch.int32, device="cuda")
        ctx.adaptive_budgets(d, n, k, s, alpha, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().reshape(L, H)
    for l in range(L):
        want = orc.adaptive_budgets(scores[l].astype(np.float64), k, s, alpha)
        assert got[l].tolist() == want.tolist(), (l, k, s, alpha)
    return got


@pytest.mark.parametrize("H,n", [(8, 4096 + 37), (8, 300), (3, 1000), (1, 500), (16, 700), (40, 257)])
def test_adaptive_budgets_random_scores(gu, H, n):
    rng = np.random.default_rng([H, n])
    sc = (rng.lognormal(0.0, 2.0, size=(3, H, n)) * rng.lognormal(0, 1, size=(3, H, 1))).astype(np.float32)
    sc /= sc.sum(-1, keepdims=True)
    for (k, s, alpha) in [(n // 10, 4, 0.2), (n // 2, 4, 0.2), (n // 5, 0, 0.0), (n // 5, 4, 1.0),
                          (n, 4, 0.2), (n - 1, 4, 0.5), (3, 4, 0.2), (0, 4, 0.2), (n // 3, n + 7, 0.2)]:
        _ada_case(gu, sc, k, s, alpha)


def test_adaptive_budgets_ties_across_heads(gu):
    rng = np.random.default_rng(31)
    H, n = 8, 2000
    sc = (rng.integers(1, 5, size=(2, H, n)) / 64.0).astype(np.float32)       # few distinct values
    sc[1, 3] = 0.25                                                            # one head entirely tied
    sc[1, 5, 10:] = 0.0
    for (k, s, alpha) in [(200, 4, 0.2), (1000, 4, 0.2), (500, 0, 0.0), (1999, 4, 0.1)]:
        _ada_case(gu, sc, k, s, alpha)


@pytest.mark.parametrize("H,n", [(512, 70), (1024, 41), (100, 300)])
def test_adaptive_budgets_many_heads(gu, H, n):
    # far more KV heads per layer than any GQA model has: the per-head digit histograms of the
    # allocation's last step then take fewer bits per level (the header allows up to 1024 heads)
    rng = np.random.default_rng([H, n, 5])
    sc = rng.lognormal(0.0, 1.5, size=(2, H, n)).astype(np.float32)
    sc /= sc.sum(-1, keepdims=True)
    sc[1, :, : n // 2] = np.round(sc[1, :, : n // 2] * 64) / 64 + np.float32(1e-3)   # ties across heads
    for (k, s, alpha) in [(n // 4, 4, 0.2), (n // 2, 0, 0.0), (n - 1, 2, 0.5)]:
        _ada_case(gu, sc, k, s, alpha)


def test_adaptive_budgets_random_distributions(gu):
    # Seeded sweep over shapes and score distributions: continuous, heavily tied (multiples of
    # 1/8), a wide range with scores of 2 and above (the last bin), nine tenths of a head equal
    # (a bin too full for the lists), and strongly skewed.  Given scores: exact.  Both the
    # allocating entry point and the one on the static workspace.
    import torch
    rng = np.random.default_rng(20250915)
    for case in range(60):
        L = int(rng.integers(1, 10)); H = int(rng.choice([1, 2, 3, 8, 16, 40, 100])); n = int(rng.integers(2, 3000))
        if case % 10 == 0:
            L, H, n = int(rng.integers(1, 4)), int(rng.choice([2, 8])), int(rng.integers(20000, 70000))
        kind = case % 5
        x = rng.random((L, H, n))
        if kind == 0: sc = x
        elif kind == 1: sc = np.round(x * 8) / 8
        elif kind == 2: sc = np.exp(rng.normal(0, 3, (L, H, n)))
        elif kind == 3: sc = np.where(x < 0.9, 0.25, x)
        else: sc = x ** 8
        sc = sc.astype(np.float32) if kind == 2 else (sc / sc.sum(-1, keepdims=True)).astype(np.float32)
        s = int(rng.choice([0, 1, 4, 64])); k = int(rng.integers(0, n + 1))
        alpha = float(rng.choice([0.0, 0.1, 0.2, 0.5, 0.9, 1.0]))
        print(f"  case {case}: L{L} H{H} n{n} kind{kind} k{k} s{s} alpha{alpha}", flush=True)
        with B.Context(L, H, 4, 128, 64, "bf16", n, 1) as ctx:
            d = torch.from_numpy(sc).cuda()
            out = torch.full((L * H,), -1, dtype=torch.int32, device="cuda")
            out2 = torch.full((L * H,), -1, dtype=torch.int32, device="cuda")
            ctx.adaptive_budgets(d, n, k, s, alpha, out)
            ctx.adaptive_budgets_noalloc(d, n, k, s, alpha, out2)
            torch.cuda.synchronize()
            assert torch.equal(out, out2)
            got = out.cpu().numpy().reshape(L, H)
        for l in range(L):
            want = orc.adaptive_budgets(sc[l].astype(np.float64), k, s, alpha)
            assert got[l].tolist() == want.tolist(), (case, l)


def test_adaptive_budgets_general_routes(gu):
    # inputs that the usual route of the allocation hands to its general one: a layer whose
    # scores are (nearly) all equal, so that the bin holding the threshold is too full for
    # the key lists; scores of 2 and above, which all share the last bin; and both at once
    rng = np.random.default_rng(77)
    H, n = 8, 6000
    sc = np.empty((4, H, n), dtype=np.float32)
    sc[0] = 1.0 / n                                                                # all equal
    sc[1] = (1.0 + rng.integers(0, 4, size=(H, n)) * 2.0 ** -23).astype(np.float32) / n   # last-bit ties, one bin
    sc[2] = rng.lognormal(3.0, 1.0, size=(H, n)).astype(np.float32) + 2.0        # everything >= 2
    sc[3] = rng.lognormal(0.0, 3.0, size=(H, n)).astype(np.float32)              # straddles 2
    sc[3, 2] = 5.0
    for (k, s, alpha) in [(n // 10, 4, 0.2), (n // 3, 0, 0.0), (n - 5, 4, 0.3)]:
        _ada_case(gu, sc, k, s, alpha)


def test_adaptive_end_to_end_c3_shape(gu):
    # scores -> adaptive budgets -> select -> compact, the selection being the layer-wide one
    import torch
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=4, n=3000 + 11)
    K, V = wl.host_cache(cfg)
    L, H, n = cfg.layers, cfg.kv_heads, cfg.n
    k, s, alpha = int(0.1 * n), 4, 0.2
    Kd, Vd = gu.to_device(K, "bf16"), gu.to_device(V, "bf16")
    with B.Context(L, H, 4, 128, cfg.r, "bf16", n, cfg.sketch_seed) as ctx:
        sc = torch.empty((L * H, n), dtype=torch.float32, device="cuda")
        ctx.scores(Kd, Vd, n, sc)
        bd = torch.empty((L * H,), dtype=torch.int32, device="cuda")
        ctx.adaptive_budgets(sc, n, k, s, alpha, bd)
        torch.cuda.synchronize()
        budgets = bd.cpu().numpy()
        sc_h = sc.cpu().numpy()
        # the allocation against the oracle's, made from the oracle's own scores
        for l in range(L):
            lt = np.stack([orc.scores(orc.to_f64(K[l, h], "bf16"), orc.to_f64(V[l, h], "bf16"),
                                      orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, "bf16")) for h in range(H)])
            gu.check_adaptive_budgets(budgets[l * H:(l + 1) * H], lt, k, s, alpha, where=f"layer {l}")
        assert np.all(budgets.reshape(L, H).sum(1) == H * k) and budgets.min() >= int(alpha * k)
        assert len(set(budgets.tolist())) > 1                                   # it does adapt
        off = wl.offsets_for(budgets)
        idx = torch.empty((int(off[-1]),), dtype=torch.int32, device="cuda")
        Ko = torch.empty((int(off[-1]), 128), dtype=torch.bfloat16, device="cuda"); Vo = torch.empty_like(Ko)
        ctx.select(sc, n, budgets, s, off, idx)
        ctx.compact(Kd, Vd, n, idx, off, Ko, Vo)
        torch.cuda.synchronize()
        idx_h, Ko_h, Vo_h = idx.cpu().numpy(), gu.to_host(Ko, "bf16"), gu.to_host(Vo, "bf16")
    for l in range(L):
        for h in range(H):
            i = l * H + h
            G = orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, "bf16")
            a, b = int(off[i]), int(off[i + 1])
            gu.check_head(cfg, None, K[l, h], V[l, h], G, sc_h[i], idx_h[a:b], Ko_h[a:b], Vo_h[a:b],
                          int(budgets[i]), s, where=f"ada l{l} h{h}")


@pytest.mark.parametrize("layers,kv_heads,n,r,dtype", [(32, 8, 2000 + 11, 64, "bf16"),   # fused scoring phases
                                                        (2, 4, 5000 + 3, 128, "bf16"),   # general kernels
                                                        (3, 2, 40000 + 1, 32, "bf16"),   # streaming selection
                                                        (1, 8, 700, 32, "fp32")])
def test_adaptive_one_call_on_device(gu, layers, kv_heads, n, r, dtype):
    # scores -> budgets -> offsets -> select -> gather in one call, nothing through the host
    import torch
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=layers, kv_heads=kv_heads, n=n, r=r, dtype=dtype)
    K, V = wl.host_cache(cfg)
    L, H = cfg.layers, cfg.kv_heads
    heads = L * H
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Kd, Vd = gu.to_device(K, dtype), gu.to_device(V, dtype)
    lt_layers = [np.stack([orc.scores(orc.to_f64(K[l, h], dtype), orc.to_f64(V[l, h], dtype),
                                      orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, dtype)) for h in range(H)])
                 for l in range(L)]
    with B.Context(L, H, 4, 128, cfg.r, dtype, n, cfg.sketch_seed) as ctx:
        for (k, s, alpha) in [(n // 10, 4, 0.2), (n // 3, 0, 0.0), (n // 20, 64, 1.0), (3, 4, 0.2), (0, 4, 0.2)]:
            total = heads * k
            # every output between canaries: budgets, offsets and the block table are made on the
            # device here, so an overrun would not be caught by any host-side check
            guards = {"scores": gu.Guarded((heads, n), torch.float32, float("nan")),
                      "budgets": gu.Guarded((heads,), torch.int32, -7),
                      "offsets": gu.Guarded((heads + 1,), torch.int64, -7),
                      "indices": gu.Guarded((max(total, 1),), torch.int32, -1),
                      "K_out": gu.Guarded((max(total, 1), 128), tdt, 0.0),
                      "V_out": gu.Guarded((max(total, 1), 128), tdt, 0.0)}
            sc, bd, od, idx, Ko, Vo = (guards[w].t for w in ("scores", "budgets", "offsets", "indices", "K_out", "V_out"))
            ctx.compress_adaptive(Kd, Vd, n, k, s, alpha, sc, bd, od, idx, Ko, Vo)
            torch.cuda.synchronize()
            for what, g in guards.items():
                g.check(f"compress_adaptive k{k} s{s} a{alpha}: {what}")
            budgets, off, sc_h = bd.cpu().numpy(), od.cpu().numpy(), sc.cpu().numpy()
            for l in range(L):        # against the oracle's allocation, made from the oracle's own scores
                gu.check_adaptive_budgets(budgets[l * H:(l + 1) * H], lt_layers[l], k, s, alpha,
                                          where=f"k{k} s{s} a{alpha} layer {l}")
            assert off.tolist() == wl.offsets_for(budgets).tolist() and off[-1] == total
            idx_h, Ko_h, Vo_h = idx.cpu().numpy(), gu.to_host(Ko, dtype), gu.to_host(Vo, dtype)
            for l in range(L):
                for h in range(H):
                    i = l * H + h
                    G = orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, dtype)
                    a, b = int(off[i]), int(off[i + 1])
                    gu.check_head(cfg, None, K[l, h], V[l, h], G, sc_h[i], idx_h[a:b], Ko_h[a:b], Vo_h[a:b],
                                  int(budgets[i]), s, where=f"ada one call k{k} s{s} a{alpha} l{l} h{h}")
        # without a score buffer of the caller's
        # (fresh buffers of the right size: the loop above ended with the empty budget)
        k, s, alpha = n // 10, 4, 0.2
        idx = torch.empty((heads * k,), dtype=torch.int32, device="cuda")
        Ko = torch.empty((heads * k, 128), dtype=tdt, device="cuda"); Vo = torch.empty_like(Ko)
        bd2 = torch.empty((heads,), dtype=torch.int32, device="cuda")
        od2 = torch.empty((heads + 1,), dtype=torch.int64, device="cuda")
        idx2 = torch.empty((heads * k,), dtype=torch.int32, device="cuda")
        Ko2 = torch.empty((heads * k, 128), dtype=tdt, device="cuda"); Vo2 = torch.empty_like(Ko2)
        ctx.compress_adaptive(Kd, Vd, n, k, s, alpha, sc, bd, od, idx, Ko, Vo)
        ctx.compress_adaptive(Kd, Vd, n, k, s, alpha, None, bd2, od2, idx2, Ko2, Vo2)
        torch.cuda.synchronize()
        assert torch.equal(bd, bd2) and torch.equal(od, od2) and torch.equal(idx, idx2)
        ity = torch.int16 if dtype == "bf16" else torch.int32
        assert torch.equal(Ko.view(ity), Ko2.view(ity)) and torch.equal(Vo.view(ity), Vo2.view(ity))
        # every rejected call returns before anything is launched
        for args in [(Kd, Vd, n, n + 1, 4, 0.2, sc, bd, od, idx, Ko, Vo), (Kd, Vd, n, 5, 4, 1.2, sc, bd, od, idx, Ko, Vo),
                     (Kd, Vd, n, 5, 4, 0.2, sc, None, od, idx, Ko, Vo), (Kd, Vd, n, 5, 4, 0.2, sc, bd, None, idx, Ko, Vo),
                     (Kd, Vd, n, 5, 4, 0.2, sc, bd, od, None, Ko, Vo), (Kd, Vd, n + 1, 5, 4, 0.2, sc, bd, od, idx, Ko, Vo)]:
            with pytest.raises(B.CurdkvError) as e:
                ctx.compress_adaptive(*args)
            assert e.value.code == B.ERR_INVALID_ARG


def test_adaptive_one_call_with_a_safeguarded_head(gu):
    # one head of every layer has identical rows, hence equal scores 1/n: next to the peaked
    # heads of its layer it stays below the layer's threshold and is kept alive by the safeguard
    # alone.  Its selection cannot take the layer's threshold over and searches its own (among
    # equal keys: the lowest token numbers), while the other heads of the layer do take it over.
    import torch
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=32, n=3000 + 7)          # 256 heads: fused scoring phases
    K, V = wl.host_cache(cfg)
    L, H, n = cfg.layers, cfg.kv_heads, cfg.n
    for l in range(L):
        K[l, l % H] = K[l, l % H, 0]
        V[l, l % H] = V[l, l % H, 0]
    heads = L * H
    k, s, alpha = n // 8, 4, 0.2
    Kd, Vd = gu.to_device(K, "bf16"), gu.to_device(V, "bf16")
    with B.Context(L, H, 4, 128, cfg.r, "bf16", n, cfg.sketch_seed) as ctx:
        assert ctx.uses_fused_kernel(n)
        sc = torch.empty((heads, n), dtype=torch.float32, device="cuda")
        bd = torch.empty((heads,), dtype=torch.int32, device="cuda")
        od = torch.empty((heads + 1,), dtype=torch.int64, device="cuda")
        idx = torch.full((heads * k,), -1, dtype=torch.int32, device="cuda")
        Ko = torch.zeros((heads * k, 128), dtype=torch.bfloat16, device="cuda"); Vo = torch.zeros_like(Ko)
        ctx.compress_adaptive(Kd, Vd, n, k, s, alpha, sc, bd, od, idx, Ko, Vo)
        torch.cuda.synchronize()
        budgets, off, sc_h, idx_h = bd.cpu().numpy(), od.cpu().numpy(), sc.cpu().numpy(), idx.cpu().numpy()
        Ko_h, Vo_h = gu.to_host(Ko, "bf16"), gu.to_host(Vo, "bf16")
    g = int(np.floor(alpha * k))
    for l in range(L):
        lt = np.stack([orc.scores(orc.to_f64(K[l, h], "bf16"), orc.to_f64(V[l, h], "bf16"),
                                  orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, "bf16")) for h in range(H)])
        gu.check_adaptive_budgets(budgets[l * H:(l + 1) * H], lt, k, s, alpha, where=f"layer {l}")
        flat = l * H + l % H
        assert budgets[flat] == g, (l, budgets[l * H:(l + 1) * H])        # the safeguard, sinks included
        assert idx_h[off[flat]:off[flat + 1]].tolist() == list(range(g))  # equal scores: lowest tokens
        for h in range(H):
            i = l * H + h
            a, b = int(off[i]), int(off[i + 1])
            gu.check_head(cfg, None, K[l, h], V[l, h], None, sc_h[i], idx_h[a:b], Ko_h[a:b], Vo_h[a:b],
                          int(budgets[i]), s, where=f"l{l} h{h}", lt=lt[h])


def test_adaptive_budgets_errors(gu):
    import torch
    with B.Context(1, 2, 4, 128, 64, "bf16", 64, 1) as ctx:
        sc = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
        out = torch.zeros((2,), dtype=torch.int32, device="cuda")
        for args in [(sc, 64, 65, 4, 0.2, out), (sc, 64, -1, 4, 0.2, out), (sc, 64, 10, 4, 1.5, out),
                     (sc, 64, 10, -1, 0.2, out), (None, 64, 10, 4, 0.2, out), (sc, 64, 10, 4, 0.2, None),
                     (sc, 65, 10, 4, 0.2, out)]:
            with pytest.raises(B.CurdkvError) as e:
                ctx.adaptive_budgets(*args)
            assert e.value.code == B.ERR_INVALID_ARG


# ---- scoring during generation: chunk by chunk, then the usual selection -----------------

@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_incremental_scoring_matches_full_cache(gu, dtype):
    import torch
    cfg = wl.scaled(wl.CONFIGS["c2"], layers=2, kv_heads=3, n=1500 + 9, dtype=dtype)
    K, V = wl.host_cache(cfg)
    L, H, n = cfg.layers, cfg.kv_heads, cfg.n
    heads, cap = L * H, 2048
    chunks = [700, 1, 1, 63, 300, 1, n - 1066]            # prefill, single decode steps, ragged chunks
    assert sum(chunks) == n
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    with B.Context(L, H, 4, 128, cfg.r, dtype, cap, cfg.sketch_seed) as ctx:
        raw = torch.full((heads, cap), float("nan"), dtype=torch.float32, device="cuda")
        sums = torch.full((heads,), float("nan"), dtype=torch.float64, device="cuda")
        done = 0
        for m in chunks:
            Kc = gu.to_device(np.ascontiguousarray(K[:, :, done:done + m]), dtype)
            Vc = gu.to_device(np.ascontiguousarray(V[:, :, done:done + m]), dtype)
            ctx.scores_append(Kc, Vc, m, done, cap, raw, sums)
            done += m
            if done in (700, 702, n):                     # compress at several points of the stream
                sc = torch.empty((heads, done), dtype=torch.float32, device="cuda")
                ctx.normalise(raw, sums, cap, done, sc)
                b = np.full(heads, done // 5, dtype=np.int32); off = wl.offsets_for(b)
                idx = torch.empty((int(off[-1]),), dtype=torch.int32, device="cuda")
                Kd = gu.to_device(np.ascontiguousarray(K[:, :, :done]), dtype)
                Vd = gu.to_device(np.ascontiguousarray(V[:, :, :done]), dtype)
                Ko = torch.empty((int(off[-1]), 128), dtype=tdt, device="cuda"); Vo = torch.empty_like(Ko)
                ctx.select(sc, done, b, 4, off, idx)
                ctx.compact(Kd, Vd, done, idx, off, Ko, Vo)
                torch.cuda.synchronize()
                sc_h, idx_h = sc.cpu().numpy(), idx.cpu().numpy()
                Ko_h, Vo_h = gu.to_host(Ko, dtype), gu.to_host(Vo, dtype)
                for l in range(L):
                    for h in range(H):
                        i = l * H + h
                        G = orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, dtype)
                        a, e = int(off[i]), int(off[i + 1])
                        gu.check_head(cfg, None, K[l, h, :done], V[l, h, :done], G, sc_h[i], idx_h[a:e],
                                      Ko_h[a:e], Vo_h[a:e], int(b[i]), 4, where=f"incremental n={done} l{l} h{h}")
        # rows beyond the scored ones were never touched
        assert bool(torch.isnan(raw[:, n:]).all())
        # argument checks
        for args in [(Kc, Vc, 0, 0, cap, raw, sums), (Kc, Vc, 5, cap - 4, cap, raw, sums),
                     (Kc, Vc, 5, 0, cap + 1, raw, sums), (None, Vc, 5, 0, cap, raw, sums)]:
            with pytest.raises(B.CurdkvError):
                ctx.scores_append(*args)


# ---- randomised shapes and adversarial score distributions --------------------------------

def test_random_small_shapes_both_paths(gu):
    rng = np.random.default_rng(2024)
    for case in range(36):
        L = int(rng.integers(1, 4)); H = int(rng.choice([1, 2, 3, 8])); n = int(rng.integers(1, 700 if case < 24 else 5000))
        r = int(rng.choice([8, 20, 32, 64, 128])); s = int(rng.choice([0, 1, 4, 9]))
        dtype = "bf16" if case % 4 else "fp32"
        cfg = wl.scaled(wl.CONFIGS["c2"], layers=L, kv_heads=H, n=n, r=r, dtype=dtype)
        b = rng.integers(0, n + 1, size=L * H).astype(np.int32)
        source = ["kv", "kv", "k", "v"][case % 4 if case >= 12 else 0]
        projection = not (case >= 12 and case % 3 == 0)
        print(f"  case {case}: L{L} H{H} n{n} r{r} s{s} {dtype} {source} projection={projection}", flush=True)
        gu.run_and_check(cfg, b, n_sink=s, one_call=bool(case % 2), source=source, projection=projection)
    for case in range(6):                                  # enough heads for the fused kernel
        n = int(rng.integers(1, 400)); r = int(rng.choice([20, 32, 64])); s = int(rng.choice([0, 4, 50]))
        cfg = wl.scaled(wl.CONFIGS["c3"], n=n, r=r)
        b = rng.integers(0, n + 1, size=256).astype(np.int32)
        print(f"  fused case {case}: n{n} r{r} s{s}", flush=True)
        gu.run_and_check(cfg, b, n_sink=s, one_call=True, fused=True)


@pytest.mark.parametrize("n", [5000, 33000, 36000, 36864, 50000])
def test_select_adversarial_scores(gu, n):
    # huge dynamic range, denormals, zeros, blocks of duplicates straddling the cut: every
    # variant of the selection kernel (registers for n <= 36864, streaming above) must agree
    # with the oracle exactly, since the scores are given and ties go by index
    import torch
    rng = np.random.default_rng(n)
    H, s = 6, 4
    sc = np.empty((H, n), dtype=np.float32)
    sc[0] = np.exp2(rng.uniform(-140, 120, size=n)).astype(np.float32)          # incl. denormals
    sc[1] = 0.0; sc[1, rng.choice(n, 50, replace=False)] = 1e-30                # almost all zero
    sc[2] = rng.choice(np.array([1e-3, 2e-3, 3e-3], dtype=np.float32), size=n)  # three values
    sc[3] = np.float32(1.0) + rng.integers(0, 3, size=n).astype(np.float32) * np.float32(2.0 ** -23)  # last-bit ties
    sc[4] = np.sort(rng.random(n).astype(np.float32))                            # ascending
    sc[5] = np.sort(rng.random(n).astype(np.float32))[::-1]                      # descending
    for budgets in ([n // 10] * H, [n - 1, 5, n // 2, n // 3, 1, n], [0, 4, 3, n // 7, n // 2, n // 2]):
        b = np.array(budgets, dtype=np.int32); off = wl.offsets_for(b)
        with B.Context(1, H, 4, 128, 64, "bf16", n, 1) as ctx:
            idx = torch.full((max(int(off[-1]), 1),), -1, dtype=torch.int32, device="cuda")
            ctx.select(torch.from_numpy(sc).cuda(), n, b, s, off, idx)
            torch.cuda.synchronize()
            idx = idx.cpu().numpy()
        for h in range(H):
            want = orc.select(sc[h].astype(np.float64), int(b[h]), s)
            assert np.array_equal(idx[off[h]:off[h + 1]], want), (n, h, budgets)


def _one_full_bin(rng, n, in_bin):
    """Scores whose cut falls into a bin of the selection's 4096-bin histogram that holds exactly
    `in_bin` keys: that many values 1 + i*2^-23 (one bin: 32 bins per binade), some of them equal,
    a few thousand larger values, the rest spread far below."""
    sc = (rng.random(n).astype(np.float32) * np.float32(0.4) + np.float32(1e-3))
    where = rng.permutation(n)
    sc[where[:in_bin]] = np.float32(1.0) + (rng.integers(0, max(in_bin // 3, 2), size=in_bin)).astype(np.float32) * np.float32(2.0 ** -23)
    big = where[in_bin:in_bin + n // 50]
    sc[big] = np.float32(1.5) + rng.random(big.size).astype(np.float32) * np.float32(0.4)
    return sc, n // 50


@pytest.mark.parametrize("n,in_bin", [(20000, 9999), (20000, 10000), (20000, 10001),      # registers: list of cap/2 = n/2 pairs
                                      (36864, 16384), (36864, 16385),                     # cap bounded by LDS: 32768 words
                                      (100000, 8192), (100000, 8193), (131072, 8000)])    # streaming: 8192 pairs
def test_select_bin_capacity_boundaries(gu, n, in_bin):
    # the usual route of the selection lists the keys inside the cut bin; a bin that holds one
    # key more than the list takes goes the general route: both sides of every capacity, exact
    import torch
    rng = np.random.default_rng([n, in_bin])
    H, s = 3, 4
    sc = np.empty((H, n), dtype=np.float32)
    budgets = []
    for h in range(H):
        sc[h], above = _one_full_bin(rng, n, in_bin)
        budgets.append(s + above + [1, in_bin // 2, in_bin][h])       # cut at the top, middle and bottom of the bin
    b = np.array(budgets, dtype=np.int32); off = wl.offsets_for(b)
    with B.Context(1, H, 4, 128, 64, "bf16", n, 1) as ctx:
        idx = torch.full((int(off[-1]),), -1, dtype=torch.int32, device="cuda")
        ctx.select(torch.from_numpy(sc).cuda(), n, b, s, off, idx)
        torch.cuda.synchronize()
        idx = idx.cpu().numpy()
    for h in range(H):
        want = orc.select(sc[h].astype(np.float64), int(b[h]), s)
        assert np.array_equal(idx[off[h]:off[h + 1]], want), (n, in_bin, h)


@pytest.mark.parametrize("per_head", [511, 512, 513, 2048, 2049])
def test_adaptive_list_capacity_boundaries(gu, per_head):
    # the allocation's last workgroup resolves up to 4096 keys of the layer's cut bin in LDS
    # (8 heads x 512) and each head hands in up to 2048: one key beyond either takes the general route
    rng = np.random.default_rng(per_head)
    H, n, s = 8, 12000, 4
    sc = np.empty((2, H, n), dtype=np.float32)
    for l in range(2):
        for h in range(H):
            sc[l, h], above = _one_full_bin(rng, n, per_head)
    k = s + n // 50 + per_head // 2                      # the layer's cut lands inside the full bins
    for alpha in (0.0, 0.2):
        _ada_case(gu, sc, k, s, alpha)


def test_eviction_loss_of_the_gpu_selection(gu):
    # What the selection is for (Section 3.1, Lemma 1; Figures 1 and 2), on the index sets the HIP
    # path returns: the evaluator's eviction loss of the GPU's set equals that of the oracle's set
    # wherever the two sets are the same, Lemma 1's inequality holds for the GPU's set, and the
    # value-guided choice keeps far more of the value mass than as many random tokens would.
    from oracle import eviction_eval as ev
    for (layers, kv_heads, one_call, fused) in [(1, 4, False, False), (32, 8, True, True)]:
        cfg = wl.scaled(wl.CONFIGS["c2"], layers=layers, kv_heads=kv_heads, n=1024)
        K, V = wl.host_cache(cfg)
        L, H, n, s = cfg.layers, cfg.kv_heads, cfg.n, 4
        k = n // 10
        budgets = np.full(L * H, k, dtype=np.int32)
        with B.Context(L, H, 4, 128, cfg.r, "bf16", n, cfg.sketch_seed) as ctx:
            assert ctx.uses_fused_kernel(n) == fused
            _, idx, _, _, off = gu.run_path(ctx, gu.to_device(K, "bf16"), gu.to_device(V, "bf16"), n, budgets, s,
                                            "bf16", one_call)
            idx = idx.cpu().numpy().astype(np.int64)
        rng = np.random.default_rng(21)
        same = 0
        groups = [(l, h) for l in range(L) for h in range(H)][:: max(1, L * H // 8)]      # eight groups at most
        for (l, h) in groups:
            i = l * H + h
            S_gpu = idx[off[i]:off[i + 1]]
            K64, V64 = orc.to_f64(K[l, h], "bf16"), orc.to_f64(V[l, h], "bf16")
            lt = orc.scores(K64, V64, orc.sketch(cfg.sketch_seed, l, h, H, 128, cfg.r, "bf16"))
            S_orc = orc.select(lt, k, s)
            Q = K64[rng.choice(n, 16, replace=False)] * 0.5 + rng.standard_normal((16, 128)) * 0.5
            loss_gpu, loss_orc = ev.eviction_loss(Q, K64, V64, S_gpu), ev.eviction_loss(Q, K64, V64, S_orc)
            if np.array_equal(S_gpu, S_orc):
                assert loss_gpu == loss_orc
                same += 1
            else:                                    # near-cut ties only (checked elsewhere): a few tokens' worth
                assert abs(loss_gpu - loss_orc) <= 0.05 * loss_orc
            assert loss_gpu > 0.0 and ev.eviction_loss(Q, K64, V64, np.arange(n)) < 1e-9
            lhs, rhs = ev.lemma1_sides(Q, K64, V64, S_gpu)
            assert lhs <= rhs
            vn = np.sum(V64 * V64, axis=1)
            assert vn[S_gpu].sum() / vn.sum() > 0.3                                  # random keeps 0.1 on average
            rnd = np.mean([np.sqrt(vn.sum() - vn[rng.choice(n, k, replace=False)].sum()) for _ in range(5)])
            assert np.sqrt(vn.sum() - vn[S_gpu].sum()) < 0.9 * rnd                   # Lemma 1's ||V - V'||_F term
        assert same >= len(groups) - 1


def test_fold_gqa(gu):
    import torch
    L, H, g, n = 2, 3, 4, 1000
    rng = np.random.default_rng(13)
    sq = rng.random((L * H, g, n)).astype(np.float32)
    sq[0] = sq[0, 0]                                 # CurDKV case: the group shares one score
    with B.Context(L, H, g, 128, 64, "bf16", n, 1) as ctx:
        d = torch.from_numpy(sq).cuda()
        out = torch.empty((L * H, n), dtype=torch.float32, device="cuda")
        ctx.fold(d, n, out)
        torch.cuda.synchronize()
        out = out.cpu().numpy()
    assert np.array_equal(out[0], sq[0, 0])          # identity, bit for bit
    for i in range(L * H):
        want = orc.fold_gqa(sq[i].astype(np.float64))
        assert np.allclose(out[i], want, rtol=1e-6, atol=0)


def test_user_supplied_sketch(gu):
    cfg = wl.scaled(wl.CONFIGS["c2"], kv_heads=2, n=500)
    import torch
    K, V = wl.host_cache(cfg)
    rng = np.random.default_rng(14)
    Gs = [rng.standard_normal((128, cfg.r)).astype(np.float32) / 8.0 for _ in range(2)]
    with B.Context(1, 2, 4, 128, cfg.r, "bf16", cfg.n, 5) as ctx:
        for h in range(2):
            ctx.set_sketch(0, h, Gs[h])
        sc = torch.empty((2, cfg.n), dtype=torch.float32, device="cuda")
        ctx.scores(gu.to_device(K, "bf16"), gu.to_device(V, "bf16"), cfg.n, sc)
        torch.cuda.synchronize()
        sc = sc.cpu().numpy()
    for h in range(2):
        G = orc.round_to_storage(Gs[h].astype(np.float64), "bf16")
        lt = orc.scores(orc.to_f64(K[0, h], "bf16"), orc.to_f64(V[0, h], "bf16"), G)
        gu.check_scores(sc[h], lt, f"user sketch h{h}")


def test_repeatable_bitwise(gu):
    import torch
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=2, n=3000)
    K, V = wl.host_cache(cfg)
    Kd, Vd = gu.to_device(K, "bf16"), gu.to_device(V, "bf16")
    b = wl.budgets_for(cfg, 0.2)
    outs = []
    for _ in range(2):
        with B.Context(cfg.layers, cfg.kv_heads, 4, 128, cfg.r, "bf16", cfg.n, cfg.sketch_seed) as ctx:
            sc, idx, Ko, Vo, _ = gu.run_path(ctx, Kd, Vd, cfg.n, b, 4, "bf16")
            outs.append((sc.clone(), idx.clone(), Ko.clone(), Vo.clone()))
    for a, c in zip(*outs):
        assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                           c.view(torch.int32) if c.dtype == torch.float32 else c)


def test_error_paths_launch_nothing(gu):
    import torch
    n, H = 64, 2
    with B.Context(1, H, 4, 128, 64, "bf16", n, 1) as ctx:
        K = torch.zeros((H, n, 128), dtype=torch.bfloat16, device="cuda")
        sc = torch.zeros((H, n), dtype=torch.float32, device="cuda")
        idx = torch.zeros((2 * n,), dtype=torch.int32, device="cuda")
        good_b = np.array([8, 8], dtype=np.int32)
        good_o = wl.offsets_for(good_b)

        def code(fn, *a):
            with pytest.raises(B.CurdkvError) as e:
                fn(*a)
            return e.value.code

        assert code(ctx.scores, K, K, n + 1, sc) == B.ERR_INVALID_ARG       # n > max_tokens
        assert code(ctx.scores, K, K, 0, sc) == B.ERR_INVALID_ARG
        assert code(ctx.scores, None, K, n, sc) == B.ERR_INVALID_ARG
        assert code(ctx.scores, K.data_ptr() + 2, K, n, sc) == B.ERR_INVALID_ARG   # misaligned
        assert code(ctx.select, sc, n, np.array([8, n + 1], dtype=np.int32), 4,
                    wl.offsets_for(np.array([8, n + 1])), idx) == B.ERR_INVALID_ARG
        assert code(ctx.select, sc, n, np.array([8, -1], dtype=np.int32), 4,
                    np.array([0, 8, 7], dtype=np.int64), idx) == B.ERR_INVALID_ARG
        assert code(ctx.select, sc, n, good_b, 4, np.array([0, 8, 17], dtype=np.int64), idx) == B.ERR_INVALID_ARG
        assert code(ctx.select, sc, n, good_b, 4, np.array([1, 9, 17], dtype=np.int64), idx) == B.ERR_INVALID_ARG
        assert code(ctx.select, sc, n, good_b, -1, good_o, idx) == B.ERR_INVALID_ARG
        assert code(ctx.select, sc, n, good_b, 4, good_o, None) == B.ERR_INVALID_ARG
        assert code(ctx.compact, K, K, n, idx, np.array([0, 8, 8 + n + 1], dtype=np.int64), K, K) == B.ERR_INVALID_ARG
        assert code(ctx.compact, K, K, n, None, good_o, K, K) == B.ERR_INVALID_ARG
        # out-of-range indices are skipped by the kernel, never dereferenced
        bad = torch.tensor([0, 1, 2, 3, -5, 10 ** 6, 6, 7] * 2, dtype=torch.int32, device="cuda")
        Ko = torch.zeros((16, 128), dtype=torch.bfloat16, device="cuda")
        Vo = torch.zeros((16, 128), dtype=torch.bfloat16, device="cuda")
        ctx.compact(K, K, n, bad, good_o, Ko, Vo)
        torch.cuda.synchronize()
    with pytest.raises(B.CurdkvError) as e:
        B.Context(1, 1, 1, 64, 64, "bf16", 16, 1)
    assert e.value.code == B.ERR_UNSUPPORTED


# ---- HIP graphs: the compute calls only enqueue kernels, so a graph can hold them ------------

@pytest.mark.parametrize("layers,n,one_call", [(32, 2000 + 17, True), (1, 3000 + 5, True), (2, 1500, False)])
def test_graph_capture_and_replay(gu, layers, n, one_call):
    # captured once, replayed on fresh data with eager work and synchronisations in between;
    # every replay must give, bit for bit, what the eager call gives on the same inputs
    import torch
    cfg = wl.scaled(wl.CONFIGS["c3"], layers=layers, n=n)
    heads = layers * cfg.kv_heads
    budgets = wl.budgets_for(cfg, 0.1)
    off = wl.offsets_for(budgets)
    total = int(off[-1])
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)

    def fresh():
        return (torch.randn((heads, n, 128), device="cuda", generator=gen) *
                torch.rand((heads, n, 1), device="cuda", generator=gen)).to(torch.bfloat16)

    Kd, Vd = fresh(), fresh()
    sc = torch.empty((heads, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((total,), dtype=torch.int32, device="cuda")
    Ko = torch.empty((total, 128), dtype=torch.bfloat16, device="cuda"); Vo = torch.empty_like(Ko)
    with B.Context(layers, cfg.kv_heads, 4, 128, cfg.r, "bf16", n, cfg.sketch_seed) as ctx:
        def call():
            if one_call:
                ctx.compress(Kd, Vd, n, budgets, 4, off, sc, idx, Ko, Vo)
            else:
                ctx.scores(Kd, Vd, n, sc)
                ctx.select(sc, n, budgets, 4, off, idx)
                ctx.compact(Kd, Vd, n, idx, off, Ko, Vo)
        call()                                   # before the capture: uploads the offsets
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call()
        for rep in range(3):
            Kd.copy_(fresh()); Vd.copy_(fresh())
            for t in (sc, idx, Ko, Vo):
                t.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = [t.clone() for t in (sc, idx, Ko.view(torch.int16), Vo.view(torch.int16))]
            for t in (sc, idx, Ko, Vo):
                t.zero_()
            call()
            torch.cuda.synchronize()
            for a, b in zip(got, (sc, idx, Ko.view(torch.int16), Vo.view(torch.int16))):
                assert torch.equal(a, b), rep
            assert int(idx.max()) < n and float(sc.sum()) > 0.99 * heads
        del g


# ---- one context reused: smaller n than max_tokens, changing budgets, other streams, two contexts ----

def test_context_reuse_changing_sizes_budgets_and_streams(gu):
    import torch
    big = wl.scaled(wl.CONFIGS["c3"], layers=2, kv_heads=4, n=3000)
    other = wl.scaled(wl.CONFIGS["c4"], layers=1, kv_heads=3, n=777, r=32)
    Kb, Vb = wl.host_cache(big)
    Ko_, Vo_ = wl.host_cache(other)
    side = torch.cuda.Stream()
    rng = np.random.default_rng(77)
    with B.Context(2, 4, 4, 128, big.r, "bf16", big.n, big.sketch_seed) as ctx, \
         B.Context(1, 3, 4, 128, other.r, "bf16", 1000, other.sketch_seed) as ctx2:
        def run(c, cfg, K, V, n, budgets, s, stream, one_call):
            # the first n tokens of every head, contiguous
            Kd = gu.to_device(np.ascontiguousarray(K[:, :, :n]), "bf16")
            Vd = gu.to_device(np.ascontiguousarray(V[:, :, :n]), "bf16")
            heads = cfg.layers * cfg.kv_heads
            off = wl.offsets_for(budgets); tot = int(off[-1])
            sc = torch.empty((heads, n), dtype=torch.float32, device="cuda")
            idx = torch.full((max(tot, 1),), -1, dtype=torch.int32, device="cuda")
            Ko = torch.full((max(tot, 1), 128), float("nan"), dtype=torch.bfloat16, device="cuda"); Vo = Ko.clone()
            torch.cuda.synchronize()
            st = stream if stream is not None else torch.cuda.current_stream()
            if one_call:
                c.compress(Kd, Vd, n, budgets, s, off, sc, idx, Ko, Vo, stream=st)
            else:
                c.scores(Kd, Vd, n, sc, stream=st)
                c.select(sc, n, budgets, s, off, idx, stream=st)
                c.compact(Kd, Vd, n, idx, off, Ko, Vo, stream=st)
            st.synchronize()
            sc_h, idx_h, Ko_h, Vo_h = sc.cpu().numpy(), idx.cpu().numpy(), gu.to_host(Ko, "bf16"), gu.to_host(Vo, "bf16")
            for l in range(cfg.layers):
                for h in range(cfg.kv_heads):
                    i = l * cfg.kv_heads + h
                    G = orc.sketch(cfg.sketch_seed, l, h, cfg.kv_heads, 128, cfg.r, "bf16")
                    a, b = int(off[i]), int(off[i + 1])
                    gu.check_head(cfg, None, K[l, h, :n], V[l, h, :n], G, sc_h[i], idx_h[a:b], Ko_h[a:b], Vo_h[a:b],
                                  int(budgets[i]), s, where=f"reuse n={n} l{l} h{h}")
        uniform = np.full(8, 300, dtype=np.int32)
        for step in range(10):
            n = int(rng.choice([big.n, 1234, 64, 2999, 1]))
            budgets = uniform.clip(max=n) if step % 3 == 0 else rng.integers(0, n + 1, size=8).astype(np.int32)
            run(ctx, big, Kb, Vb, n, budgets, int(rng.choice([0, 4, 64])), side if step % 2 else None, bool(step % 4 < 2))
            if step % 3 == 1:                    # the other context in between, its own plan and sketches
                n2 = int(rng.choice([other.n, 100]))
                run(ctx2, other, Ko_, Vo_, n2, rng.integers(0, n2 + 1, size=3).astype(np.int32), 4, None, True)


def test_generation_loop_compress_append_compress(gu):
    # Section 3.2: compression during generation.  A cache is compressed after the prompt, grows
    # token by token, and is compressed again whenever it passes a limit; the library scores only
    # the new rows each step and re-scores the kept rows after a compression.  The oracle runs
    # the same loop on its own copy of the cache, re-scoring everything each time.
    import torch
    cfg = wl.scaled(wl.CONFIGS["c2"], layers=1, kv_heads=4, n=1100)
    K, V = wl.host_cache(cfg)                                   # the token stream: prompt, then generated tokens
    H, cap, limit, keep, s = 4, 1024, 320, 256, 4
    prompt = 600
    Gs = [orc.sketch(cfg.sketch_seed, 0, h, H, 128, cfg.r, "bf16") for h in range(H)]
    # oracle's cache, per head: arrays of rows (storage bits)
    oK = [K[0, h, :prompt].copy() for h in range(H)]
    oV = [V[0, h, :prompt].copy() for h in range(H)]
    with B.Context(1, H, 4, 128, cfg.r, "bf16", cap, cfg.sketch_seed) as ctx:
        Kc = torch.zeros((H, cap, 128), dtype=torch.bfloat16, device="cuda"); Vc = torch.zeros_like(Kc)
        raw = torch.zeros((H, cap), dtype=torch.float32, device="cuda")
        sums = torch.zeros((H,), dtype=torch.float64, device="cuda")
        n = prompt
        Kc[:, :n] = gu.to_device(np.ascontiguousarray(K[0, :, :n]), "bf16")
        Vc[:, :n] = gu.to_device(np.ascontiguousarray(V[0, :, :n]), "bf16")
        ctx.scores_append(Kc[:, :n].contiguous(), Vc[:, :n].contiguous(), n, 0, cap, raw, sums)
        nxt, compressions = prompt, 0
        while True:
            if n >= limit:                                      # ---- compress to `keep` tokens per head
                budgets = np.full(H, keep, dtype=np.int32); off = wl.offsets_for(budgets)
                Kd, Vd = Kc[:, :n].contiguous(), Vc[:, :n].contiguous()
                sc = torch.empty((H, n), dtype=torch.float32, device="cuda")
                idx = torch.empty((H * keep,), dtype=torch.int32, device="cuda")
                Ko = torch.full((H * keep, 128), float("nan"), dtype=torch.bfloat16, device="cuda"); Vo = Ko.clone()
                ctx.normalise(raw, sums, cap, n, sc)
                ctx.select(sc, n, budgets, s, off, idx)
                ctx.compact(Kd, Vd, n, idx, off, Ko, Vo)
                torch.cuda.synchronize()
                sc_h, idx_h = sc.cpu().numpy(), idx.cpu().numpy()
                Ko_h, Vo_h = gu.to_host(Ko, "bf16"), gu.to_host(Vo, "bf16")
                for h in range(H):
                    a, b = h * keep, (h + 1) * keep
                    _, nd = gu.check_head(cfg, None, oK[h], oV[h], Gs[h], sc_h[h], idx_h[a:b], Ko_h[a:b], Vo_h[a:b],
                                          keep, s, where=f"generation loop, compression {compressions}, head {h}")
                    assert nd == 0, "a near-cut difference: the two caches would part ways (pick another seed)"
                    S = orc.select(orc.scores(orc.to_f64(oK[h], "bf16"), orc.to_f64(oV[h], "bf16"), Gs[h]), keep, s)
                    oK[h], oV[h] = orc.compact(oK[h], oV[h], S)
                n = keep
                Kc[:, :n] = Ko.view(H, keep, 128); Vc[:, :n] = Vo.view(H, keep, 128)
                ctx.scores_append(Kc[:, :n].contiguous(), Vc[:, :n].contiguous(), n, 0, cap, raw, sums)   # kept rows, afresh
                compressions += 1
                if compressions == 4:
                    break
            m = 1 if (nxt % 7) else 5                           # mostly single tokens, now and then a few
            Kn = gu.to_device(np.ascontiguousarray(K[0, :, nxt:nxt + m]), "bf16")
            Vn = gu.to_device(np.ascontiguousarray(V[0, :, nxt:nxt + m]), "bf16")
            Kc[:, n:n + m] = Kn; Vc[:, n:n + m] = Vn
            ctx.scores_append(Kn, Vn, m, n, cap, raw, sums)
            for h in range(H):
                oK[h] = np.concatenate([oK[h], K[0, h, nxt:nxt + m]]); oV[h] = np.concatenate([oV[h], V[0, h, nxt:nxt + m]])
            n += m; nxt += m
        assert nxt > prompt + 150 and compressions == 4


def test_graph_capture_adaptive_one_call(gu):
    # the adaptive one-call path is nine launches and no host round trip: it fits a graph too
    import torch
    layers, H, n, k = 4, 8, 2500, 300
    heads = layers * H
    gen = torch.Generator(device="cuda")
    gen.manual_seed(9)

    def fresh():
        return (torch.randn((heads, n, 128), device="cuda", generator=gen) *
                torch.rand((heads, n, 1), device="cuda", generator=gen)).to(torch.bfloat16)

    Kd, Vd = fresh(), fresh()
    sc = torch.empty((heads, n), dtype=torch.float32, device="cuda")
    bd = torch.empty((heads,), dtype=torch.int32, device="cuda")
    od = torch.empty((heads + 1,), dtype=torch.int64, device="cuda")
    idx = torch.empty((heads * k,), dtype=torch.int32, device="cuda")
    Ko = torch.empty((heads * k, 128), dtype=torch.bfloat16, device="cuda"); Vo = torch.empty_like(Ko)
    outs = (sc, bd, od, idx, Ko, Vo)
    with B.Context(layers, H, 4, 128, 64, "bf16", n, 3) as ctx:
        def call():
            ctx.compress_adaptive(Kd, Vd, n, k, 4, 0.2, sc, bd, od, idx, Ko, Vo)
        call()                                   # before the capture: allocates the workspaces
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call()
        for rep in range(3):
            Kd.copy_(fresh()); Vd.copy_(fresh())
            for t in outs:
                t.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = [t.clone() for t in (sc, bd, od, idx, Ko.view(torch.int16), Vo.view(torch.int16))]
            for t in outs:
                t.zero_()
            call()
            torch.cuda.synchronize()
            for a, b in zip(got, (sc, bd, od, idx, Ko.view(torch.int16), Vo.view(torch.int16))):
                assert torch.equal(a, b), rep
            assert int(od[-1]) == heads * k and len(set(bd.tolist())) > 1
        del g
