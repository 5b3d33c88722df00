"""Parity of the packed (two codes per byte) index against the CPU oracle, through the C ABI:
stored bytes and norms bit-exact against the storage definition, search results bit-exact
against the oracle's exhaustive search over the saturated codes.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

from paper_2110_08919_amd import synth

pytestmark = pytest.mark.gpu

BASES = {"skewed": synth.SKEWED_1M, "aniso": synth.ANISO_1M2, "scaled": synth.SCALED_10M,
         "product": synth.PRODUCT_100M, "tiny": synth.TINY}


@pytest.fixture(scope="module")
def lpq():
    from paper_2110_08919_amd import lpq as m
    assert torch.cuda.is_available(), "no GPU visible"
    m.lib()
    return m


def _oracle_quant(oracle, gq):
    k, sb, se, m = gq.get_params()
    oq = oracle.Quantizer(gq.d, gq.bits).set_params(k, sb, se)
    assert np.array_equal(oq.m, m)
    return oq


def _padded_features(d):
    return next(p for p in (64, 96, 128, 192, 256) if d <= p)


def _build(lpq, oracle, w, bits, mode, scope):
    x, q = w.corpus(), w.queries()
    xd = x.cuda()
    gq = lpq.Quantizer(w.d, bits).calibrate(xd, mode, scope)
    idx = lpq.Index(gq, w.n, packed=True).add_f32(xd)
    assert idx.size == w.n
    oq = _oracle_quant(oracle, gq)
    ocodes = oracle.nibble_codes(oq.encode(x.numpy()))
    oqcodes = oracle.nibble_codes(oq.encode(q.numpy()))
    return idx, gq, q, ocodes, oqcodes


@pytest.mark.parametrize("name,n,bits,mode,scope", [
    ("tiny", 3001, 4, "minmax", "per_feature"),      # d = 128; min/max calibration reaches the top code + 8
    ("aniso", 2050, 4, "absmax", "global"),          # d = 100 -> 128 features per row
    ("scaled", 1000, 3, "absmax", "global"),         # d = 96
    ("product", 777, 2, "absmax", "per_feature"),    # d = 256
])
def test_packed_rows_and_norms_bit_exact(lpq, oracle, name, n, bits, mode, scope):
    w = BASES[name].scaled(n=n, nq=4)
    idx, gq, q, ocodes, _ = _build(lpq, oracle, w, bits, mode, scope)
    rows, norms = idx.storage()
    d_pad = _padded_features(w.d)
    assert rows.shape == (n, d_pad // 2)
    assert np.array_equal(rows, oracle.pack_nibbles(ocodes, d_pad))
    assert np.array_equal(norms, (ocodes.astype(np.int64) ** 2).sum(axis=1).astype(np.int32))
    if bits == 4 and mode == "minmax":
        # the case the saturation exists for is present in the data
        raw = _oracle_quant(oracle, gq).encode(w.corpus().numpy())
        assert int(raw.max()) == 8 and int(ocodes.max()) == 7


@pytest.mark.parametrize("name,n,nq,k,metric,bits,mode,scope", [
    ("tiny", 10000, 100, 10, "l2sq", 4, "minmax", "per_feature"),     # two query tiles, the second ragged
    ("skewed", 70001, 16, 10, "l2sq", 4, "minmax", "global"),         # ragged last stage, seeding pass
    ("skewed", 140000, 5, 16, "l2sq", 4, "minmax", "per_feature"),    # largest k; three staging chunks on add
    ("aniso", 66000, 64, 10, "ip", 4, "absmax", "global"),            # d = 100, inner product: per-query term
    ("aniso", 12345, 130, 1, "ip", 3, "absmax", "global"),            # three tiles
    ("scaled", 90000, 33, 10, "l2sq", 4, "absmax", "global"),         # d = 96
    ("product", 50000, 20, 10, "ip", 4, "absmax", "per_feature"),     # d = 256: 128-byte rows
    ("product", 9000, 70, 16, "l2sq", 2, "absmax", "per_feature"),    # 2 bits: ties everywhere
    ("tiny", 40, 3, 1, "ip", 4, "absmax", "global"),                  # fewer items than one stage
    ("tiny", 300, 200, 16, "l2sq", 4, "minmax", "global"),
])
def test_packed_search_bit_exact(lpq, oracle, name, n, nq, k, metric, bits, mode, scope):
    w = BASES[name].scaled(n=n, nq=nq)
    idx, gq, q, ocodes, oqcodes = _build(lpq, oracle, w, bits, mode, scope)
    ids, dists = idx.search(q.cuda(), k, metric)
    torch.cuda.synchronize()
    oids, odists = oracle.search_i8(ocodes, oqcodes, k, metric, threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists)
    assert np.array_equal(ids.cpu().numpy(), oids)
    # the same through the entry point that takes codes (unsaturated ones: the library saturates)
    raw_q = _oracle_quant(oracle, gq).encode(q.numpy())
    ids2, dists2 = idx.search(torch.from_numpy(raw_q).cuda(), k, metric)
    torch.cuda.synchronize()
    assert torch.equal(ids2, ids) and torch.equal(dists2, dists)


@pytest.mark.parametrize("d,metric,bits", [(33, "l2sq", 4), (64, "ip", 4), (65, "l2sq", 3), (129, "ip", 4),
                                           (200, "l2sq", 4), (256, "l2sq", 4), (1, "l2sq", 4)])
def test_packed_search_every_row_length(lpq, oracle, d, metric, bits):
    """Feature counts on both sides of every padded row length (64, 96, 128, 192, 256 features)."""
    g = torch.Generator().manual_seed(d)
    n, nq, k = 30011, 70, 10
    x = torch.randn(n, d, generator=g)
    q = torch.randn(nq, d, generator=g)
    gq = lpq.Quantizer(d, bits).calibrate(x.cuda(), "absmax", "global")
    idx = lpq.Index(gq, n, packed=True).add_f32(x.cuda())
    oq = _oracle_quant(oracle, gq)
    ocodes = oracle.nibble_codes(oq.encode(x.numpy()))
    oqcodes = oracle.nibble_codes(oq.encode(q.numpy()))
    rows, norms = idx.storage()
    assert np.array_equal(rows, oracle.pack_nibbles(ocodes, _padded_features(d)))
    ids, dists = idx.search(q.cuda(), k, metric)
    torch.cuda.synchronize()
    oids, odists = oracle.search_i8(ocodes, oqcodes, k, metric, threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists)
    assert np.array_equal(ids.cpu().numpy(), oids)


@pytest.mark.parametrize("name,n,nq,k,metric,bits,mode,scope,path,region_cap", [
    ("skewed", 150_001, 700, 10, "l2sq", 4, "minmax", "global", 0, 0),       # d = 128: 128 queries per wave, ragged tiles
    ("skewed", 100_000, 300, 16, "l2sq", 4, "minmax", "per_feature", 0, 0),  # largest k
    ("aniso", 120_000, 513, 10, "ip", 4, "absmax", "global", 0, 0),          # d = 100, inner product: per-query term
    ("scaled", 90_000, 129, 1, "l2sq", 3, "absmax", "global", 0, 0),         # d = 96: three 16-byte chunks per row; smallest batch
    ("product", 80_000, 400, 10, "ip", 4, "absmax", "per_feature", 0, 0),    # d = 256: 64 queries per wave
    ("product", 70_000, 300, 10, "l2sq", 2, "absmax", "per_feature", 0, 0),  # 2 bits: ties everywhere
    ("skewed", 100_000, 300, 10, "l2sq", 4, "minmax", "global", 0, 2),       # regions of two: further rounds, then the generic kernel
    ("aniso", 66_000, 300, 10, "ip", 4, "absmax", "global", 1, 0),           # the generic kernel on packed rows
    ("skewed", 30_000, 40, 10, "l2sq", 4, "minmax", "global", 1, 0),
])
def test_packed_search_large_batches(lpq, oracle, name, n, nq, k, metric, bits, mode, scope, path, region_cap):
    """More than 128 queries on a packed index take ONE collecting scan over all queries instead of
    tiles of 64 (rows of 48 bytes or more); the generic kernel reads packed rows too (forced here,
    and the last resort of the collecting scan)."""
    w = BASES[name].scaled(n=n, nq=nq)
    idx, gq, q, ocodes, oqcodes = _build(lpq, oracle, w, bits, mode, scope)
    lpq.set_tuning(lpq.TUNE_PATH, path)
    lpq.set_tuning(lpq.TUNE_REGION_CAP, region_cap)
    try:
        ids, dists = idx.search(q.cuda(), k, metric)
        torch.cuda.synchronize()
        redone, fill = idx.overflow_stats(nq, k, metric)
        left = idx.overflow_left(nq, k, metric)
    finally:
        lpq.set_tuning(lpq.TUNE_PATH, 0)
        lpq.set_tuning(lpq.TUNE_REGION_CAP, 0)
    oids, odists = oracle.search_i8(ocodes, oqcodes, k, metric, threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists)
    assert np.array_equal(ids.cpu().numpy(), oids)
    print("flagged:", redone, "left for the generic kernel:", left, "largest region fill:", fill)
    if region_cap:
        assert redone > 16 and left > 0, (redone, left, fill)
    elif path == 0 and nq > 128:
        assert fill > 0      # the collecting scan ran


@pytest.mark.parametrize("name,n,nq,k,metric,bits", [
    ("skewed", 120_000, 5, 17, "l2sq", 4),       # one row-split tile, collecting scan
    ("skewed", 200_000, 64, 100, "l2sq", 4),
    ("aniso", 150_000, 100, 32, "ip", 4),        # 65 .. 128 queries: one scan over all of them
    ("product", 100_000, 300, 128, "ip", 3),     # d = 256, largest k
    ("tiny", 9_000, 130, 50, "l2sq", 4),         # too few items to sample: generic kernel on packed rows
])
def test_packed_search_long_lists(lpq, oracle, name, n, nq, k, metric, bits):
    """k > 16 on a packed index: the collecting scan at every batch size."""
    w = BASES[name].scaled(n=n, nq=nq)
    idx, gq, q, ocodes, oqcodes = _build(lpq, oracle, w, bits, "absmax" if metric == "ip" else "minmax", "global")
    ids, dists = idx.search(q.cuda(), k, metric)
    torch.cuda.synchronize()
    oids, odists = oracle.search_i8(ocodes, oqcodes, k, metric, threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists)
    assert np.array_equal(ids.cpu().numpy(), oids)


def test_packed_search_long_lists_on_short_rows_in_tiles(lpq, oracle):
    """d <= 64 (32 packed bytes per row) has no scan over more than 64 queries: tiles of 64, each a
    row-split collecting scan."""
    g = torch.Generator().manual_seed(5)
    n, nq, k, d = 150_000, 150, 40, 50
    x, q = torch.randn(n, d, generator=g), torch.randn(nq, d, generator=g)
    gq = lpq.Quantizer(d, 4).calibrate(x.cuda(), "absmax", "global")
    idx = lpq.Index(gq, n, packed=True).add_f32(x.cuda())
    oq = _oracle_quant(oracle, gq)
    ocodes, oqcodes = oracle.nibble_codes(oq.encode(x.numpy())), oracle.nibble_codes(oq.encode(q.numpy()))
    ids, dists = idx.search(q.cuda(), k, "l2sq")
    torch.cuda.synchronize()
    oids, odists = oracle.search_i8(ocodes, oqcodes, k, "l2sq", threads=16)
    assert np.array_equal(dists.cpu().numpy(), odists)
    assert np.array_equal(ids.cpu().numpy(), oids)


@pytest.mark.parametrize("name,n,nq,m,metric,bits", [
    ("skewed", 50_000, 37, 100, "l2sq", 4), ("aniso", 20_000, 64, 7, "ip", 4), ("product", 9_000, 5, 300, "l2sq", 3),
    ("scaled", 30_000, 20, 33, "ip", 4)])
def test_packed_gather_distances_bit_exact(lpq, oracle, name, n, nq, m, metric, bits):
    """Distances to listed items on a packed index: those of the stored nibble codes and of the
    query codes saturated the same way (handed in unsaturated), including absent ids."""
    w = BASES[name].scaled(n=n, nq=nq)
    idx, gq, q, ocodes, oqcodes = _build(lpq, oracle, w, bits, "absmax" if metric == "ip" else "minmax", "per_feature")
    r = np.random.default_rng(n + m)
    ids = r.integers(0, n, size=(nq, m), dtype=np.int32)
    ids[0, 0], ids[-1, -1] = -1, n            # "no item"
    raw_q = _oracle_quant(oracle, gq).encode(q.numpy())
    got = idx.gather_dist(torch.from_numpy(raw_q).cuda(), torch.from_numpy(ids).cuda(), metric).cpu().numpy()
    assert np.array_equal(got, oracle.gather_dist(ocodes, oqcodes, np.where(ids >= n, -1, ids), metric))


def test_packed_equals_unpacked_index_of_saturated_codes_and_incremental_add(lpq, oracle):
    w = synth.SKEWED_1M.scaled(n=100_000, nq=48)
    x, q = w.corpus().cuda(), w.queries().cuda()
    gq = lpq.Quantizer(w.d, 4).calibrate(x, "minmax", "global")
    codes = gq.encode(x)
    sat = codes.clamp(-8, 7)
    plain = lpq.Index(gq, w.n).add_i8(sat)
    packed = lpq.Index(gq, w.n, packed=True)
    packed.add_i8(codes[:33_333]).add_f32(x[33_333:70_000]).add_i8(sat[70_000:])
    assert packed.size == w.n
    qc = gq.encode(q).clamp(-8, 7)
    for metric in ("l2sq", "ip"):
        a = plain.search(qc, 10, metric)
        b = packed.search(q, 10, metric)
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    # half the bytes per row
    assert packed.data()[1] * 2 == plain.data()[1]


def test_packed_error_codes(lpq):
    w = synth.TINY.scaled(n=500, nq=4)
    x, q = w.corpus().cuda(), w.queries().cuda()
    g8 = lpq.Quantizer(w.d, 8).calibrate(x, "minmax", "per_feature")
    with pytest.raises(lpq.LpqError) as e:
        lpq.Index(g8, 500, packed=True)
    assert e.value.code == lpq.EINVAL                     # more than 4 bits
    wide = torch.randn(64, 300, device="cuda")
    gw = lpq.Quantizer(300, 4).calibrate(wide, "minmax", "per_feature")
    with pytest.raises(lpq.LpqError) as e:
        lpq.Index(gw, 64, packed=True)
    assert e.value.code == lpq.ERANGE                     # more than 256 features
    g4 = lpq.Quantizer(w.d, 4).calibrate(x, "minmax", "per_feature")
    idx = lpq.Index(g4, 500, packed=True).add_f32(x)
    with pytest.raises(lpq.LpqError) as e:
        idx.search(q, 129, "l2sq")
    assert e.value.code == lpq.ERANGE                     # k beyond what the packed scans collect
    assert idx.workspace_bytes(4, 129) == 0
