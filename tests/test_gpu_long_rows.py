"""The matrix-core collecting scan for long rows and its seeding pass (rows of 257 to 1536 features,
and large batches on rows of 192 and 256 bytes) against the CPU oracle, bit-exact on ids and int32
distances.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

from paper_2110_08919_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lpq():
    from paper_2110_08919_amd import lpq as m
    assert torch.cuda.is_available(), "no GPU visible"
    m.lib()
    return m


def _workload(recipe, d, n, nq, metric):
    return synth.Workload(f"{recipe}_x{d}", recipe, n, d, nq, metric, (10,), "minmax", "global", 3)


def _case(lpq, oracle, w, k, metric, mode, scope, expect_collecting=True):
    x, q = w.corpus("cuda"), w.queries("cuda")
    gq = lpq.Quantizer(w.d, 8).calibrate(x, mode, scope)
    index = lpq.Index(gq, w.n).add_f32(x)
    ws = torch.empty(index.workspace_bytes(w.nq, k, metric) + 256, dtype=torch.uint8, device="cuda")
    ids, dists = index.search(q, k, metric, workspace=ws)
    torch.cuda.synchronize()
    kk, sb, se, _ = gq.get_params()
    oq = oracle.Quantizer(gq.d, gq.bits).set_params(kk, sb, se)
    oids, odists = oracle.search_i8(oq.encode(x.cpu().numpy()), oq.encode(q.cpu().numpy()), k, metric, threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists)
    assert np.array_equal(ids.cpu().numpy(), oids)
    if expect_collecting:
        _, fill = index.overflow_stats(w.nq, k, metric, ws)
        assert fill > 0, "the collecting scan was expected to run here"
    return index, ws


@pytest.mark.parametrize("recipe,d,n,nq,k,metric,mode,scope", [
    ("bimodal", 300, 70_003, 130, 10, "l2sq", "minmax", "per_feature"),   # padded to 384, ragged tail
    ("scaled_unit", 384, 66_000, 5, 10, "ip", "absmax", "global"),
    ("skewed_int", 500, 80_000, 1030, 100, "l2sq", "minmax", "global"),   # padded to 512, k = 100; eight-wave workgroups
    ("bimodal", 512, 90_011, 64, 10, "ip", "absmax", "per_feature"),
    ("scaled_unit", 700, 70_000, 129, 17, "l2sq", "absmax", "global"),    # padded to 768
    ("bimodal", 768, 100_000, 700, 10, "l2sq", "minmax", "per_feature"),  # eight-wave workgroups
    ("scaled_unit", 1000, 66_000, 513, 10, "ip", "absmax", "global"),
    ("skewed_int", 960, 65_536, 33, 128, "l2sq", "minmax", "global"),     # padded to 1024, largest k of the scan
    ("bimodal", 1024, 75_001, 1, 10, "ip", "absmax", "global"),
    ("scaled_unit", 1100, 66_000, 200, 10, "l2sq", "absmax", "global"),   # padded to 1536: three segments per row
    ("skewed_int", 1536, 70_003, 700, 100, "l2sq", "minmax", "per_feature"),
    ("bimodal", 1536, 66_000, 33, 17, "ip", "absmax", "global"),
])
def test_search_long_rows(lpq, oracle, recipe, d, n, nq, k, metric, mode, scope):
    _case(lpq, oracle, _workload(recipe, d, n, nq, metric), k, metric, mode, scope)


@pytest.mark.parametrize("recipe,d,n,nq,k,metric,mode,scope", [
    ("bimodal", 256, 70_000, 2000, 100, "ip", "absmax", "per_feature"),
    ("skewed_int", 256, 80_003, 1900, 10, "l2sq", "minmax", "global"),
    ("scaled_unit", 180, 66_000, 2048, 16, "l2sq", "absmax", "global"),   # padded to 192
    ("bimodal", 192, 90_000, 3000, 40, "ip", "absmax", "global"),
    ("bimodal", 256, 66_000, 5200, 10, "l2sq", "minmax", "global"),       # six tiles of 1024: query rows padded beyond a multiple of 512
])
def test_search_large_batches_on_rows_of_192_and_256_bytes(lpq, oracle, recipe, d, n, nq, k, metric, mode, scope):
    """Large batches on rows of 192 and 256 bytes take the same scan with 128 queries per wave."""
    assert lpq.search_plan_info(d, 8, 0, n, nq, k)[3] == 128, "the 128-queries-per-wave tile was expected here"
    assert lpq.search_plan_info(d, 8, 0, n, 1100, k)[3] == 64, "a batch that would mostly pad its tiles keeps the 64-query tile"
    _case(lpq, oracle, _workload(recipe, d, n, nq, metric), k, metric, mode, scope)


@pytest.mark.parametrize("d", [384, 1024])
def test_search_long_rows_overflow_is_redone_exactly(lpq, oracle, d):
    """A sample far too small for k = 100: queries whose regions overflow go through the further
    rounds of the scan (and what still overflows through the generic kernel) and come back exact."""
    lpq.set_tuning(lpq.TUNE_SEED_ROWS, 8192)
    try:
        _case(lpq, oracle, _workload("skewed_int", d, 200_000, 70 if d == 384 else 600, "l2sq"), 100, "l2sq", "minmax", "global")
    finally:
        lpq.set_tuning(lpq.TUNE_SEED_ROWS, 0)


def test_search_long_rows_extreme_codes(lpq, oracle):
    """Codes at the ends of the range in 1024 dimensions: the largest dot products and norms the
    long-row scan meets, on a corpus large enough for its seeding pass."""
    d, n = 1024, 70_000
    rng = np.random.default_rng(21)
    c = rng.choice(np.array([-128, 127], np.int8), size=(n, d))
    q = rng.choice(np.array([-128, 127], np.int8), size=(40, d))
    gq = lpq.Quantizer(d, 8).set_params(np.zeros(d), np.full(d, -128.0), np.full(d, 128.0))
    idx = lpq.Index(gq, n).add_i8(torch.as_tensor(c).cuda())
    for metric in ("l2sq", "ip"):
        ids, dists = idx.search(torch.as_tensor(q).cuda(), 20, metric)
        oids, odists = oracle.search_i8(c, q, 20, metric, threads=16)
        assert np.array_equal(ids.cpu().numpy(), oids) and np.array_equal(dists.cpu().numpy(), odists)


def test_search_long_rows_small_corpus_and_large_k_take_the_generic_kernel(lpq, oracle):
    """Below the smallest sample, and for k beyond 128, long rows are searched by the generic kernel."""
    _case(lpq, oracle, _workload("bimodal", 768, 3000, 9, "l2sq"), 10, "l2sq", "minmax", "global", expect_collecting=False)
    _case(lpq, oracle, _workload("bimodal", 600, 40_000, 3, "ip"), 200, "ip", "absmax", "global", expect_collecting=False)


def _random_case(seed):
    """A random shape that the long-row scan takes: rows of 192 bytes and more, corpora large enough
    for a seeding sample, batches on both sides of the workgroup sizes and of the 1024-query tiles."""
    r = np.random.default_rng(7000 + seed)
    d = int(r.choice([180, 192, 256, 257, 300, 384, 400, 512, 513, 700, 768, 900, 1000, 1024, 1025, 1300, 1536]))
    nq = int(r.choice([1, 33, 64, 300, 512, 513, 700, 1100, 2100, 3000]))
    n = int(r.choice([33_000, 40_001, 66_000, 70_003, 100_000]))
    if d * nq * n > 8e10:                       # keep the oracle to a few seconds
        nq = max(1, int(8e10 / (d * n)))
    k = int(r.choice([1, 10, 16, 17, 40, 100, 128]))
    metric = str(r.choice(["l2sq", "ip"]))
    recipe = str(r.choice(["bimodal", "skewed_int", "scaled_unit"]))
    mode, scope = [("minmax", "per_feature"), ("minmax", "global"), ("absmax", "global")][int(r.integers(3))]
    return recipe, d, n, nq, k, metric, mode, scope


@pytest.mark.parametrize("seed", range(20))
def test_random_long_row_configuration_bit_exact(lpq, oracle, seed):
    recipe, d, n, nq, k, metric, mode, scope = _random_case(seed)
    print(dict(recipe=recipe, d=d, n=n, nq=nq, k=k, metric=metric, mode=mode, scope=scope), flush=True)
    w = synth.Workload(f"{recipe}_x{d}", recipe, n, d, nq, metric, (10,), "minmax", "global", 100 + seed)
    index, ws = _case(lpq, oracle, w, k, metric, mode, scope, expect_collecting=False)
    ids2, dists2 = index.search(w.queries("cuda"), k, metric, workspace=ws)      # the same call again: the same answer
    ids1, dists1 = index.search(w.queries("cuda"), k, metric)
    assert torch.equal(ids1, ids2) and torch.equal(dists1, dists2)


@pytest.mark.parametrize("recipe,d,n,nq,k,metric", [("bimodal", 768, 70_000, 300, 10, "l2sq"),
                                                     ("bimodal", 256, 66_000, 2000, 100, "ip"),
                                                     ("skewed_int", 1536, 40_000, 16, 17, "l2sq")])
def test_long_row_search_captured_in_a_graph_replays_exactly(lpq, recipe, d, n, nq, k, metric):
    """The long-row scan too is kernel launches only: captured in a HIP graph (after one eager call),
    every replay gives the eager result, with eager work in between."""
    w = _workload(recipe, d, n, nq, metric)
    x, q = w.corpus("cuda"), w.queries("cuda")
    index = lpq.Index(lpq.Quantizer(d, 8).calibrate(x, "minmax", "global"), n).add_f32(x)
    ids = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    dists = torch.empty_like(ids)
    ws = torch.empty(index.workspace_bytes(nq, k, metric) + 256, dtype=torch.uint8, device="cuda")

    def step():
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    step()
    torch.cuda.synchronize()
    ref_ids, ref_d = ids.clone(), dists.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for _ in range(3):
        ids.fill_(-5)
        dists.fill_(-5)
        ws.random_(0, 255)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids, ref_ids) and torch.equal(dists, ref_d)
        step()
        torch.cuda.synchronize()
        assert torch.equal(ids, ref_ids) and torch.equal(dists, ref_d)
