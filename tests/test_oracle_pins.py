"""Pins of the CPU oracle against things other than itself.

Each test ties one part of oracle/lpq_oracle.c to what the paper prints, to a closed
form, to an invariant, or to an independent numpy/scipy routine, so that a dropped
term, a wrong sign, a wrong index or a transposed operand in the oracle fails here.
All of it runs on the CPU.
"""
import itertools
import os

import numpy as np
import pytest

from paper_2110_08919_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _explicit(oracle, d, bits, k, sb, se):
    return oracle.Quantizer(d, bits).set_params(np.full(d, k, np.float32), np.full(d, sb, np.float32),
                                                np.full(d, se, np.float32))


# ---------------------------------------------------------------- worked example (Section 1)
def _read_worked_example():
    meta, pts = {}, []
    for line in open(os.path.join(GOLDEN, "worked_example_1d.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        a, b = line.split()
        if a[0].isalpha():
            meta[a] = float(b)
        else:
            pts.append((float(a), int(b)))
    return meta, pts


def test_worked_example_codes_and_neighbour(oracle):
    meta, pts = _read_worked_example()
    q = _explicit(oracle, 1, int(meta["bits"]), meta["k"], meta["S_b"], meta["S_e"])
    x = np.array([[p[0]] for p in pts], np.float32)
    codes = q.encode(x)
    assert codes[:, 0].tolist() == [p[1] for p in pts]            # {1, 2, 3, 4} as printed
    # the third point is still the nearest neighbour of the fourth
    ids, dists = oracle.search_i8(codes[:3], codes[3:4], 1, "l2sq")
    assert ids[0, 0] == int(meta["nn_of_last"]) and dists[0, 0] == 1
    # equality relaxation: codes 1 and 3 tie at distance 1 from code 2; the lower id wins
    others = codes[[0, 2, 3]]
    ids, dists = oracle.search_i8(others, codes[1:2], 3, "l2sq")
    assert ids[0].tolist() == [0, 1, 2] and dists[0].tolist() == [1, 1, 4]


# ---------------------------------------------------------------- Equation 1, hand-computed
def test_encode_closed_form_values(oracle):
    q = _explicit(oracle, 1, 8, 0.0, -1.0, 1.0)           # 2^8 / 2 = 128
    assert q.m[0] == 128.0
    x = np.array([0.5, -0.5, 0.25, -0.0078125, 0.0078124, 0.999, -1.0, 1.0, 1.5, -1.5, 0.0],
                 np.float32)[:, None]
    want = [64, -64, 32, -1, 0, 127, -128, 127, 127, -128, 0]
    assert q.encode(x)[:, 0].tolist() == want
    q4 = _explicit(oracle, 1, 4, 0.0, -1.0, 1.0)          # 2^4 / 2 = 8; +2^(B-1) = 8 is kept
    x = np.array([1.0, 2.0, -2.0, 0.99, -0.01, 0.13], np.float32)[:, None]
    assert q4.encode(x)[:, 0].tolist() == [8, 8, -8, 7, -1, 1]
    # an offset k that is not the centre of the range
    qk = _explicit(oracle, 1, 8, 1.0, 0.0, 4.0)           # m = 64
    x = np.array([1.0, 2.0, 0.0, 3.5, 4.0, 0.99], np.float32)[:, None]
    assert qk.encode(x)[:, 0].tolist() == [0, 64, -64, 127, 127, -1]


def test_encode_floor_not_round_and_per_feature_constants(oracle):
    q = oracle.Quantizer(3, 8).set_params([0, 10, -5], [-1, 0, -10], [1, 20, 0])
    assert q.m.tolist() == [128.0, 12.8000001907348633, 25.6000003814697266]
    x = np.array([[0.0117, 10.7, -5.03], [-0.0117, 9.3, -4.97]], np.float32)
    # floor toward minus infinity: 1.4976 -> 1, -1.4976 -> -2; 8.96 -> 8, -8.96 -> -9; ...
    assert q.encode(x).tolist() == [[1, 8, -1], [-2, -9, 0]]


def test_identity_quantizer(oracle):
    q = _explicit(oracle, 1, 8, 0.0, -128.0, 128.0)
    assert q.m[0] == 1.0
    x = np.arange(-128, 129, dtype=np.float32)[:, None]
    want = list(range(-128, 128)) + [127]
    assert q.encode(x)[:, 0].tolist() == want


def test_edges_nan_inf_constant_feature(oracle):
    q = oracle.Quantizer(2, 8).set_params([0, 3], [-1, 3], [1, 3])
    assert q.m[1] == 0.0
    x = np.array([[np.nan, 3.0], [np.inf, 100.0], [-np.inf, -100.0], [-1.0, 3.0], [1.0, np.nan]],
                 np.float32)
    assert q.encode(x).tolist() == [[0, 0], [127, 0], [-128, 0], [-128, 0], [127, 0]]
    const = np.tile(np.array([[1.0, 7.0]], np.float32), (5, 1))
    const[:, 0] = np.arange(5)
    qc = oracle.Quantizer(2, 8).calibrate(const, "minmax", "per_feature")
    assert qc.m[1] == 0.0 and np.all(qc.encode(const)[:, 1] == 0)
    with pytest.raises(ValueError):
        oracle.Quantizer(2, 8).calibrate(x, "minmax", "per_feature")


def test_monotone_per_feature(oracle):
    rng = np.random.default_rng(5)
    x = rng.normal(size=(4000, 6)).astype(np.float32) * np.array([1, 10, .1, 3, 1e-3, 50], np.float32)
    for mode, bits in itertools.product(("minmax", "absmax", "gauss"), (8, 5, 2)):
        q = oracle.Quantizer(6, bits).calibrate(x, mode, "per_feature")
        codes = q.encode(x).astype(np.int32)
        for i in range(6):
            order = np.argsort(x[:, i], kind="stable")
            assert np.all(np.diff(codes[order, i]) >= 0), (mode, bits, i)
        half = 1 << (bits - 1)
        assert codes.min() >= -half and codes.max() <= min(half, 127)


# ---------------------------------------------------------------- calibration
def test_calibrate_gauss_matches_numpy(oracle):
    rng = np.random.default_rng(1)
    x = (rng.normal(size=(3000, 5)) * [1, 2, 3, 4, 5] + [0, -1, 2, 10, -7]).astype(np.float32)
    q = oracle.Quantizer(5, 8).calibrate(x, "gauss", "per_feature", sigma_mult=1.0)
    mu = x.astype(np.float64).mean(0)
    sd = x.astype(np.float64).std(0, ddof=0)                 # maximum likelihood: 1/n
    np.testing.assert_allclose(q.k, mu, rtol=1e-6)
    np.testing.assert_allclose(q.sb, mu - sd, rtol=1e-6)
    np.testing.assert_allclose(q.se, mu + sd, rtol=1e-6)
    np.testing.assert_allclose(q.m, 256.0 / (2 * sd), rtol=1e-6)
    q3 = oracle.Quantizer(5, 8).calibrate(x, "gauss", "per_feature", sigma_mult=3.0)
    np.testing.assert_allclose(q3.se - q3.sb, 6 * sd, rtol=1e-6)
    # one mu, sigma for all dimensions (Section 4.1)
    g = oracle.Quantizer(5, 6).calibrate(x, "gauss", "global")
    flat = x.astype(np.float64).ravel()
    np.testing.assert_allclose(g.k, np.full(5, flat.mean()), rtol=1e-6)
    np.testing.assert_allclose(g.se - g.sb, np.full(5, 2 * flat.std()), rtol=1e-6)
    np.testing.assert_allclose(g.m, np.full(5, 64.0 / (2 * flat.std())), rtol=1e-6)


def test_calibrate_minmax_absmax_are_column_statistics(oracle):
    rng = np.random.default_rng(2)
    x = (rng.uniform(-1, 1, size=(500, 4)) * [1, 5, 0.1, 20] + [0, 3, 0, -30]).astype(np.float32)
    q = oracle.Quantizer(4, 8).calibrate(x, "minmax", "per_feature")
    assert np.array_equal(q.sb, x.min(0)) and np.array_equal(q.se, x.max(0))
    np.testing.assert_array_equal(q.k, ((x.min(0).astype(np.float64) + x.max(0)) / 2).astype(np.float32))
    a = oracle.Quantizer(4, 8).calibrate(x, "absmax", "per_feature")
    amax = np.abs(x).max(0)
    assert np.array_equal(a.se, amax) and np.array_equal(a.sb, -amax) and np.all(a.k == 0)
    np.testing.assert_array_equal(a.m, (256.0 / (2.0 * amax.astype(np.float64))).astype(np.float32))
    g = oracle.Quantizer(4, 8).calibrate(x, "absmax", "global")
    assert np.all(g.se == np.abs(x).max()) and np.all(g.sb == -np.abs(x).max())
    # a strided view (ld > d) reads the same columns
    wide = np.zeros((500, 7), np.float32)
    wide[:, :4] = x
    wide[:, 4:] = 1e9
    q2 = oracle.Quantizer(4, 8).calibrate(wide[:, :4], "minmax", "per_feature")
    assert np.array_equal(q2.sb, q.sb) and np.array_equal(q2.se, q.se)
    assert np.array_equal(q2.encode(wide[:, :4]), q.encode(x))


# ---------------------------------------------------------------- integer distances
def test_distance_symmetry_and_norm_identity(oracle):
    rng = np.random.default_rng(3)
    for d in (1, 3, 100, 128, 257):
        a = rng.integers(-128, 128, size=(20, d)).astype(np.int8)
        for i, j in itertools.product(range(0, 20, 3), repeat=2):
            dl, ds = oracle.dist(a[i], a[j], "l2sq"), oracle.dist(a[i], a[j], "ip")
            assert dl == oracle.dist(a[j], a[i], "l2sq") and ds == oracle.dist(a[j], a[i], "ip")
            assert dl >= 0 and (dl == 0) == bool(np.array_equal(a[i], a[j]))
            ai, aj = a[i].astype(np.int64), a[j].astype(np.int64)
            assert dl == int((ai * ai).sum() + (aj * aj).sum() - 2 * (ai * aj).sum())
            assert ds == int((ai * aj).sum())
    # extreme codes: no overflow at the largest magnitudes
    lo, hi = np.full(1000, -128, np.int8), np.full(1000, 127, np.int8)
    assert oracle.dist(lo, hi, "l2sq") == 255 * 255 * 1000
    assert oracle.dist(lo, lo, "ip") == 128 * 128 * 1000 and oracle.dist(lo, hi, "ip") == -128 * 127 * 1000


def test_encode_norms(oracle):
    x = synth.TINY.scaled(n=300).corpus().numpy()
    q = oracle.Quantizer(128, 8).calibrate(x, "minmax", "per_feature")
    codes, norms = q.encode(x, with_norms=True)
    assert np.array_equal(norms, (codes.astype(np.int64) ** 2).sum(1))


# ---------------------------------------------------------------- top-k against brute force
def _numpy_topk(keys, k):
    """keys [nq, n] smaller = nearer; stable on id via lexsort."""
    n = keys.shape[1]
    out = np.empty((keys.shape[0], k), np.int64)
    for i in range(keys.shape[0]):
        out[i] = np.lexsort((np.arange(n), keys[i]))[:k]
    return out


@pytest.mark.parametrize("metric", ["l2sq", "ip"])
def test_topk_tiny_alphabet_many_ties(oracle, metric):
    rng = np.random.default_rng(4)
    for n, d, nq, k in [(64, 4, 9, 64), (50, 2, 7, 13), (33, 1, 5, 33), (17, 3, 4, 1)]:
        c = rng.integers(-2, 3, size=(n, d)).astype(np.int8)
        q = rng.integers(-2, 3, size=(nq, d)).astype(np.int8)
        ids, dists = oracle.search_i8(c, q, k, metric)
        ci, qi = c.astype(np.int64), q.astype(np.int64)
        if metric == "l2sq":
            full = ((qi[:, None, :] - ci[None, :, :]) ** 2).sum(-1)
            keys = full
        else:
            full = qi @ ci.T
            keys = -full
        want = _numpy_topk(keys, k)
        assert np.array_equal(ids, want)
        assert np.array_equal(dists, np.take_along_axis(full, want, 1))
        # k rounds of arg-min with the chosen item struck out
        for i in range(nq):
            kk = keys[i].astype(np.float64).copy()
            for r in range(k):
                j = int(np.argmin(kk))                    # first minimum = lowest id
                assert ids[i, r] == j
                kk[j] = np.inf


def test_topk_row_permutation(oracle):
    rng = np.random.default_rng(6)
    c = rng.integers(-128, 128, size=(200, 16)).astype(np.int8)    # distinct distances w.h.p.
    q = rng.integers(-128, 128, size=(6, 16)).astype(np.int8)
    ids, dists = oracle.search_i8(c, q, 10, "l2sq")
    perm = rng.permutation(200)
    ids_p, dists_p = oracle.search_i8(c[perm], q, 10, "l2sq")
    assert np.array_equal(dists, dists_p)
    if all(len(set(r)) == 10 for r in dists.tolist()):
        assert np.array_equal(perm[ids_p], ids)


def test_self_match_and_duplicates(oracle):
    rng = np.random.default_rng(7)
    c = rng.integers(-100, 100, size=(120, 8)).astype(np.int8)
    c[77] = c[5]                                             # a duplicate row: lower id first
    ids, dists = oracle.search_i8(c, c[[5, 40, 77]], 2, "l2sq")
    assert dists[:, 0].tolist() == [0, 0, 0]
    assert ids[0].tolist() == [5, 77] and ids[1, 0] == 40 and ids[2].tolist() == [5, 77]


def test_search_handles_row_stride_and_shapes(oracle):
    rng = np.random.default_rng(8)
    big = rng.integers(-128, 128, size=(90, 40)).astype(np.int8)
    c = big[:, :24]                                          # ld = 40 > d = 24
    q = rng.integers(-128, 128, size=(3, 24)).astype(np.int8)
    ids, dists = oracle.search_i8(c, q, 5, "ip")
    full = q.astype(np.int64) @ c.astype(np.int64).T         # [3, 90]: queries are rows
    want = _numpy_topk(-full, 5)
    assert np.array_equal(ids, want) and np.array_equal(dists, np.take_along_axis(full, want, 1))


# ---------------------------------------------------------------- reduces to exact search
def test_integer_data_reduces_to_exact_search(oracle):
    """Integer features spanning [0, 255] with one global [min, max] range give
    code = x - 128, so integer distances equal the real ones and recall is 1."""
    from scipy.spatial.distance import cdist
    w = synth.SKEWED_1M.scaled(n=3000, nq=40)
    x, qf = w.corpus().numpy(), w.queries().numpy()
    x[0, 0], x[1, 0] = 0.0, 255.0                            # make the span exact
    quant = oracle.Quantizer(128, 8).calibrate(x, "minmax", "global")
    assert quant.k[0] == 127.5 and quant.m[0] == np.float32(256.0 / 255.0)
    codes, qcodes = quant.encode(x), quant.encode(qf)
    assert np.array_equal(codes.astype(np.int32), x.astype(np.int32) - 128)
    ids, dists = oracle.search_i8(codes, qcodes, 10, "l2sq", threads=4)
    real = cdist(qf.astype(np.float64), x.astype(np.float64), "sqeuclidean")
    want = _numpy_topk(real, 10)
    assert np.array_equal(ids, want)
    assert np.array_equal(dists, np.take_along_axis(real, want, 1).astype(np.int64))
    eids, edists = oracle.search_f32(x, qf, 10, "l2sq", threads=4)
    assert np.array_equal(eids, want) and oracle.recall(ids, eids) == 1.0
    assert np.array_equal(edists, np.take_along_axis(real, want, 1).astype(np.float32))


def test_exact_search_matches_cdist_and_matmul(oracle):
    from scipy.spatial.distance import cdist
    w = synth.ANISO_1M2.scaled(n=700, nq=11)
    x, q = w.corpus().numpy(), w.queries().numpy()
    ids, d = oracle.search_f32(x, q, 7, "l2sq")
    real = cdist(q.astype(np.float64), x.astype(np.float64), "sqeuclidean")
    want = _numpy_topk(real, 7)
    assert np.array_equal(ids, want)
    np.testing.assert_allclose(d, np.take_along_axis(real, want, 1), rtol=1e-6)
    ids, s = oracle.search_f32(x, q, 7, "ip")
    ip = q.astype(np.float64) @ x.astype(np.float64).T
    want = _numpy_topk(-ip, 7)
    assert np.array_equal(ids, want)
    np.testing.assert_allclose(s, np.take_along_axis(ip, want, 1), rtol=1e-6)
    assert np.all(np.diff(s, axis=1) <= 0)                   # descending inner product


# ---------------------------------------------------------------- quantization error bound
def test_code_differences_track_scaled_differences(oracle):
    """For in-range values of one feature |(c_a - c_b) - m (a - b)| < 1 (+ rounding);
    with one global m, |sqrt(D_int) - m ||a - b||| <= sqrt(d)."""
    w = synth.TINY.scaled(n=400, nq=20)
    x, q = w.corpus().numpy(), w.queries().numpy()
    quant = oracle.Quantizer(128, 8).calibrate(np.vstack([x, q]), "minmax", "global")
    cx, cq = quant.encode(x).astype(np.int64), quant.encode(q).astype(np.int64)
    m = float(quant.m[0])
    dc = cq[:, None, :] - cx[None, :, :]
    dr = m * (q[:, None, :].astype(np.float64) - x[None, :, :])
    # the stored code of the one value equal to S_e is 127 instead of 128
    assert np.abs(dc - dr).max() < 2.0 + 1e-3 and np.mean(np.abs(dc - dr) < 1.0 + 1e-3) > 0.9999
    dint = np.sqrt((dc ** 2).sum(-1))
    dreal = np.sqrt((dr ** 2).sum(-1))
    assert np.abs(dint - dreal).max() <= np.sqrt(128) + 0.1


def test_recall_definition(oracle):
    exact = np.array([[1, 2, 3, 4], [5, 6, 7, 8], [9, 10, 11, 12]], np.int32)
    approx = np.array([[4, 3, 2, 1], [5, 6, 0, 99], [13, 14, 15, 16]], np.int32)
    assert oracle.recall(approx, exact) == pytest.approx((1.0 + 0.5 + 0.0) / 3)
    assert oracle.recall(exact, exact) == 1.0


def test_tiny_workload_recall_is_plausible(oracle):
    """Not a pin (the paper prints no recall for synthetic data): int8 search with
    per-feature min/max on the narrow-band data keeps most exact neighbours."""
    w = synth.TINY.scaled(n=4000, nq=30)
    x, q = w.corpus().numpy(), w.queries().numpy()
    quant = oracle.Quantizer(128, 8).calibrate(x, "minmax", "per_feature")
    ids, _ = oracle.search_i8(quant.encode(x), quant.encode(q), 10, "l2sq", threads=4)
    eids, _ = oracle.search_f32(x, q, 10, "l2sq", threads=4)
    assert oracle.recall(ids, eids) > 0.9


# ---------------------------------------------------------------- candidate lists (gather, re-rank)
def test_gather_distances_match_numpy_and_the_search(oracle):
    """phi between a query and listed items: against numpy's direct sums, and consistent with the
    exhaustive search (the distances the search reports are the gathered ones at its ids)."""
    rng = np.random.default_rng(5)
    codes = rng.integers(-128, 128, (300, 37), dtype=np.int8)
    q = rng.integers(-128, 128, (9, 37), dtype=np.int8)
    ids = rng.integers(0, 300, (9, 17)).astype(np.int32)
    ids[2, 5] = -1
    for metric in ("l2sq", "ip"):
        got = oracle.gather_dist(codes, q, ids, metric)
        c = codes[np.maximum(ids, 0)].astype(np.int64)
        qq = q.astype(np.int64)[:, None, :]
        ref = ((c - qq) ** 2).sum(-1) if metric == "l2sq" else (c * qq).sum(-1)
        ok = ids >= 0
        assert np.array_equal(got[ok], ref[ok])
        assert got[2, 5] == (np.iinfo(np.int32).max if metric == "l2sq" else np.iinfo(np.int32).min)
        sids, sd = oracle.search_i8(codes, q, 12, metric)
        assert np.array_equal(oracle.gather_dist(codes, q, sids, metric), sd)


def test_rerank_matches_numpy_sort_and_full_candidate_list_is_exact_search(oracle):
    """Re-rank = exact fp64 distances of the listed items, sorted by (distance, id): against numpy
    lexsort on float64 sums; with every item listed it must return the exact search of cdist."""
    from scipy.spatial.distance import cdist
    rng = np.random.default_rng(6)
    x = rng.standard_normal((200, 11)).astype(np.float32)
    q = rng.standard_normal((7, 11)).astype(np.float32)
    cand = np.stack([rng.permutation(200)[:40] for _ in range(7)]).astype(np.int32)
    cand[3, 7] = -1
    for metric in ("l2sq", "ip"):
        ids, d = oracle.rerank_f32(x, q, cand, 10, metric)
        for i in range(7):
            c = cand[i][cand[i] >= 0]
            xs, qs = x[c].astype(np.float64), q[i].astype(np.float64)
            val = ((xs - qs) ** 2).sum(1) if metric == "l2sq" else -(xs @ qs)
            order = np.lexsort((c, val))[:10]
            assert np.array_equal(ids[i], c[order])
            np.testing.assert_allclose(d[i], (val[order] if metric == "l2sq" else -val[order]).astype(np.float32), rtol=1e-6)
    allc = np.tile(np.arange(200, dtype=np.int32), (7, 1))
    ids, d = oracle.rerank_f32(x, q, allc, 5, "l2sq")
    full = cdist(q.astype(np.float64), x.astype(np.float64), "sqeuclidean")
    assert np.array_equal(ids, np.argsort(full, axis=1, kind="stable")[:, :5])
    short, sd = oracle.rerank_f32(x, q, cand[:, :3], 5, "ip")      # fewer candidates than k
    assert np.all(short[:, 3:] == -1) and np.all(np.isneginf(sd[:, 3:]))


# ---------------------------------------------------------------- quantile clip (Section 4.2, outliers)
@pytest.mark.parametrize("scope", ["per_feature", "global"])
def test_quantile_clip_matches_numpy_order_statistics(oracle, scope):
    """S_b / S_e of the quantile mode are order statistics: against numpy's sort; p = 0 is [min, max]."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((501, 7)).astype(np.float32)
    x[3, 2] = 1e6                       # an outlier the clip must drop
    x[:50, 5] = 0.25                    # duplicates
    for p in (0.0, 0.01, 0.1, 0.25):
        q = oracle.Quantizer(7, 8).calibrate(x, "quantile", scope, sigma_mult=p)
        cols = [np.sort(x[:, i]) for i in range(7)] if scope == "per_feature" else [np.sort(x.ravel())] * 7
        for i, c in enumerate(cols):
            n = c.size
            lo, hi = c[int(np.floor(p * (n - 1)))], c[int(np.ceil((1.0 - p) * (n - 1)))]
            assert q.sb[i] == lo and q.se[i] == hi
            assert q.k[i] == np.float32((np.float64(lo) + np.float64(hi)) / 2.0)
        if p == 0.0:
            mm = oracle.Quantizer(7, 8).calibrate(x, "minmax", scope)
            assert np.array_equal(q.sb, mm.sb) and np.array_equal(q.se, mm.se) and np.array_equal(q.m, mm.m)
    q = oracle.Quantizer(7, 8).calibrate(x, "quantile", "per_feature", sigma_mult=0.01)
    assert q.se[2] < 10.0               # the outlier no longer sets the range


# ---------------------------------------------------------------- nibble storage (B <= 4)
def test_nibble_saturation_and_packing_by_hand(oracle):
    # every int8 value: only those outside [-8, 7] change, and they move to the nearer end
    allv = np.arange(-128, 128).astype(np.int8)
    sat = oracle.nibble_codes(allv)
    for v, s in zip(allv.tolist(), sat.tolist()):
        assert s == (7 if v > 7 else -8 if v < -8 else v)
    # bytes written out by hand: (-8, 7) -> 0x0 | 0xF << 4; (0, 0) -> 0x88; (8 -> 7, -1) -> 0xF | 0x7 << 4;
    # an odd feature count leaves the high nibble at code 0 (= 8), padding bytes are 0x88
    rows = np.array([[-8, 7, 0, 0, 8, -1, 3]], np.int8)
    packed = oracle.pack_nibbles(rows, 10)
    assert packed.tolist() == [[0xF0, 0x88, 0x7F, 0x8B, 0x88]]
    # unpacking with shifts and masks gives the saturated codes back
    rng = np.random.default_rng(5)
    c = rng.integers(-9, 10, size=(7, 13)).astype(np.int8)
    p = oracle.pack_nibbles(c, 16).astype(np.int32)
    un = np.stack([(p & 15) - 8, (p >> 4) - 8], axis=2).reshape(7, 16)
    assert np.array_equal(un[:, :13], oracle.nibble_codes(c))
    assert np.all(un[:, 13:] == 0)


# ---------------------------------------------------------------- shared-width scope (Section 3.2, last sentence)
def _offset_data(rng, n, d):
    """Dimensions with different offsets AND different spreads."""
    mu, sg = rng.uniform(-1, 1, d), rng.uniform(0.02, 0.2, d)
    return (rng.normal(size=(n, d)) * sg + mu).astype(np.float32)


@pytest.mark.parametrize("mode,arg", [("minmax", 1.0), ("quantile", 0.01), ("gauss", 2.0)])
def test_shared_width_keeps_centres_and_gives_every_dimension_the_widest_range(oracle, mode, arg):
    x = _offset_data(np.random.default_rng(11), 2000, 24)
    pf = oracle.Quantizer(24, 8).calibrate(x, mode, "per_feature", arg)
    sh = oracle.Quantizer(24, 8).calibrate(x, mode, "shared_width", arg)
    w_pf = pf.se.astype(np.float64) - pf.sb.astype(np.float64)
    w_sh = sh.se.astype(np.float64) - sh.sb.astype(np.float64)
    widest = int(np.argmax(w_pf))
    assert np.array_equal(sh.k, pf.k)                                       # offsets stay per dimension
    assert sh.sb[widest] == pf.sb[widest] and sh.se[widest] == pf.se[widest]  # the widest range is unchanged
    np.testing.assert_allclose(w_sh, w_pf.max(), rtol=1e-6)                 # one width (up to binary32 endpoints)
    c_pf = (pf.sb.astype(np.float64) + pf.se.astype(np.float64)) / 2
    c_sh = (sh.sb.astype(np.float64) + sh.se.astype(np.float64)) / 2
    np.testing.assert_allclose(c_sh, c_pf, atol=1e-6)                       # centres stay
    np.testing.assert_allclose(sh.m, sh.m[0], rtol=1e-6)                    # hence one scale


def test_shared_width_with_absmax_is_the_global_absmax(oracle):
    x = _offset_data(np.random.default_rng(12), 1500, 10)
    sh = oracle.Quantizer(10, 8).calibrate(x, "absmax", "shared_width")
    gl = oracle.Quantizer(10, 8).calibrate(x, "absmax", "global")
    assert np.array_equal(sh.sb, gl.sb) and np.array_equal(sh.se, gl.se)
    assert np.array_equal(sh.k, gl.k) and np.array_equal(sh.m, gl.m)


def test_shared_width_on_offset_integer_data_reduces_to_exact_search(oracle):
    """Integer data, dimension i spanning [o_i, o_i + r_i] with r_i odd and the widest r = 255: the
    common scale is fl32(256/255), centres are half-integers, and every code is the value shifted by
    a per-dimension integer - so integer distances equal the exact ones and the int8 search IS the
    exact search, although offsets differ by thousands.  (Per-feature scales do not have this property.)"""
    rng = np.random.default_rng(13)
    d, n, nq, k = 12, 600, 40, 7
    r = np.concatenate([[255], rng.integers(0, 127, d - 1) * 2 + 1])
    off = rng.integers(-3000, 3000, d)
    x = off + rng.integers(0, r + 1, size=(n, d))
    x[0], x[1] = off, off + r                                  # both ends observed in every dimension
    q = off + rng.integers(0, r + 1, size=(nq, d))
    xf, qf = x.astype(np.float32), q.astype(np.float32)
    qz = oracle.Quantizer(d, 8).calibrate(xf, "minmax", "shared_width")
    assert np.all(qz.m == np.float32(256.0 / 255.0))
    ids, dists = oracle.search_i8(qz.encode(xf), qz.encode(qf), k, "l2sq")
    exact = ((q[:, None, :] - x[None, :, :]) ** 2).sum(-1)     # int64, no rounding anywhere
    for i in range(nq):
        order = np.lexsort((np.arange(n), exact[i]))[:k]
        assert np.array_equal(ids[i], order)
        assert np.array_equal(dists[i], exact[i][order])
    pf = oracle.Quantizer(d, 8).calibrate(xf, "minmax", "per_feature")
    _, d_pf = oracle.search_i8(pf.encode(xf), pf.encode(qf), k, "l2sq")
    assert not np.array_equal(d_pf, dists)                     # the pin can tell the scopes apart


def test_shared_width_preserves_l2_up_to_one_step_per_dimension(oracle):
    """With one scale m the code distance tracks the real one: | sqrt(D_int) - m |a - b| | <= sqrt(d)
    for in-range points (each coordinate difference is off by less than one step)."""
    rng = np.random.default_rng(14)
    x = _offset_data(rng, 800, 16)
    qz = oracle.Quantizer(16, 8).calibrate(x, "minmax", "shared_width")
    c = qz.encode(x).astype(np.int64)
    m = float(qz.m.astype(np.float64).mean())
    a, b = rng.integers(0, 800, 300), rng.integers(0, 800, 300)
    d_int = np.sqrt(((c[a] - c[b]) ** 2).sum(1))
    d_real = np.sqrt(((x[a].astype(np.float64) - x[b].astype(np.float64)) ** 2).sum(1))
    assert np.all(np.abs(d_int - m * d_real) <= np.sqrt(16) * (1 + 1e-5))
