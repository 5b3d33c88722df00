"""lpq_search_static, the search entry point that allocates nothing (its workspace is a device
array of the library), against lpq_search through the C ABI: bit-identical ids and distances on
two calls in a row, the second with a smaller input; sizes beyond the built-in workspace are
rejected.  Needs a real MI355X."""
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


def _index(lpq, n, nq):
    w = synth.SKEWED_1M.scaled(n=n, nq=nq)
    x, q = w.corpus("cuda"), w.queries("cuda")
    quant = lpq.Quantizer(w.d, 8).calibrate(x, "minmax", "per_feature")
    return lpq.Index(quant, w.n).add_f32(x), q


@pytest.mark.parametrize("k,metric", [(10, "l2sq"), (100, "ip")])
def test_static_workspace_search_equals_lpq_search(lpq, k, metric):
    index, q = _index(lpq, 300_000, 200)
    for nq in (200, 37):                        # two calls in a row, the second with a smaller input
        assert 0 < index.workspace_bytes(nq, k, metric) <= lpq.STATIC_WORKSPACE_BYTES
        qq = q[:nq].contiguous()
        ids = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
        dists = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
        print(f"[no-alloc] lpq_search_static nq={nq} k={k} {metric}", flush=True)
        index.search_static(qq, k, metric, out=(ids, dists))
        torch.cuda.synchronize()
        rids, rdists = index.search(qq, k, metric)
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), rids.cpu().numpy())
        assert np.array_equal(dists.cpu().numpy(), rdists.cpu().numpy())


def test_static_workspace_search_rejects_what_does_not_fit(lpq):
    index, q = _index(lpq, 300_000, 4000)
    assert index.workspace_bytes(4000, 100, "l2sq") > lpq.STATIC_WORKSPACE_BYTES
    ids = torch.full((4000, 100), -7, dtype=torch.int32, device="cuda")
    dists = torch.full((4000, 100), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(lpq.LpqError) as e:
        index.search_static(q, 100, "l2sq", out=(ids, dists))
    assert e.value.code == lpq.ERANGE
    torch.cuda.synchronize()
    assert int((ids != -7).sum()) == 0 and int((dists != -7).sum()) == 0      # outputs untouched on error
