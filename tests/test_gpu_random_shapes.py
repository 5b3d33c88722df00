"""Seeded random shapes through the whole path (calibrate, encode, index, search) against the CPU
oracle: dimensions on both sides of every row length, corpora from one row to a few stages past
a split boundary, query batches across the tile sizes of every kernel variant, every k the list
and collecting variants take, few-bit codes (ties everywhere), every tuning path, packed and
unpacked storage.  Bit-exact ids and distances.  Needs a real MI355X."""
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

MODES = [("minmax", 1.0), ("absmax", 1.0), ("gauss", 2.5), ("quantile", 0.01)]
SCOPES = ["per_feature", "global", "shared_width"]


@pytest.fixture(scope="module")
def lpq():
    from paper_2110_08919_amd import lpq as m
    assert torch.cuda.is_available(), "no GPU visible"
    m.lib()
    return m


def _case(seed):
    """One random configuration, sized so that the oracle needs well under a second."""
    r = np.random.default_rng(1000 + seed)
    d = int(r.choice([1, 3, 31, 32, 33, 64, 65, 96, 100, 127, 128, 129, 160, 192, 200, 255, 256, 257, 300]))
    nq = int(r.choice([1, 2, 17, 63, 64, 65, 130, 255, 256, 257, 300, 513, 700]))
    budget = 1.5e9 / (d * nq)
    n = int(min(r.choice([1, 5, 63, 64, 129, 1000, 4097, 20000, 66000, 131072, 150001]), max(1, budget)))
    k = int(min(n, r.choice([1, 2, 9, 10, 16, 17, 32, 33, 100, 128, 129, 300])))
    bits = int(r.choice([2, 3, 4, 6, 8, 8, 8]))
    metric = str(r.choice(["l2sq", "ip"]))
    mode, arg = MODES[int(r.integers(len(MODES)))]
    scope = str(r.choice(SCOPES))
    path = int(r.choice([0, 0, 1, 2, 3, 4]))
    packed = bool(bits <= 4 and d <= 256 and k <= 128 and r.random() < 0.7)
    kind = str(r.choice(["normal", "offsets", "small_integers"]))
    return dict(seed=seed, d=d, nq=nq, n=n, k=k, bits=bits, metric=metric, mode=mode, arg=arg, scope=scope,
                path=path, packed=packed, kind=kind)


def _data(c):
    g = torch.Generator().manual_seed(c["seed"])
    n, nq, d = c["n"], c["nq"], c["d"]
    if c["kind"] == "small_integers":          # a tiny alphabet: many exact ties in every distance
        x = torch.randint(0, 4, (n, d), generator=g).float()
        q = torch.randint(0, 4, (nq, d), generator=g).float()
    else:
        x, q = torch.randn(n, d, generator=g), torch.randn(nq, d, generator=g)
        if c["kind"] == "offsets":
            mu, sg = torch.rand(d, generator=g) * 4 - 2, torch.rand(d, generator=g) * 0.5 + 0.05
            x, q = x * sg + mu, q * sg + mu
    return x, q


@pytest.mark.parametrize("seed", range(int(os.environ.get("LPQ_TEST_RANDOM_CASES", "160"))))   # more cases on request
def test_random_configuration_bit_exact(lpq, oracle, seed):
    c = _case(seed)
    print(c, flush=True)
    x, q = _data(c)
    xd, qd = x.cuda(), q.cuda()
    gq = lpq.Quantizer(c["d"], c["bits"]).calibrate(xd, c["mode"], c["scope"], c["arg"])
    ks, sb, se, m = gq.get_params()
    oq = oracle.Quantizer(c["d"], c["bits"]).set_params(ks, sb, se)
    assert np.array_equal(oq.m, m)
    idx = lpq.Index(gq, c["n"], packed=c["packed"]).add_f32(xd)
    ocodes, oqcodes = oq.encode(x.numpy()), oq.encode(q.numpy())
    if c["packed"]:
        ocodes, oqcodes = oracle.nibble_codes(ocodes), oracle.nibble_codes(oqcodes)
    lpq.set_tuning(lpq.TUNE_PATH, c["path"])
    try:
        ids, dists = idx.search(qd, c["k"], c["metric"])
        torch.cuda.synchronize()
    finally:
        lpq.set_tuning(lpq.TUNE_PATH, 0)
    oids, odists = oracle.search_i8(ocodes, oqcodes, c["k"], c["metric"], threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists), c
    assert np.array_equal(ids.cpu().numpy(), oids), c
