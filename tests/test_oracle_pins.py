"""Pins for the CPU oracle: every check here compares oracle output with something
the paper or the mathematics fixes (closed forms in float64, brute force by definition,
special cases, a hand-worked example), never with the oracle's own formula retyped.
No GPU is used."""
import os

import numpy as np
import pytest

from oracle import index_build
from paper_2508_17828_amd import synth
from tests import helpers

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def tiny(oracle):
    # C1's law and index shape at 2,000 vectors; brute-force candidates
    return helpers.cached("C1", 2000, 24)


@pytest.fixture(scope="module")
def tiny_ivf(oracle):
    # C2's law and index shape (M=32, dsub=4) at 6,000 vectors with 16 lists / 5 probes
    return helpers.cached("C2", 6000, 20, 16, 5)


def _recon(ix):
    M, dsub = ix.M, ix.d // ix.M
    r = np.empty((ix.n, ix.d), np.float64)
    for j in range(M):
        r[:, j * dsub:(j + 1) * dsub] = ix.codebooks[j][ix.codes[:, j]]
    return r


# ---- exact distance ------------------------------------------------------------------

def test_exact_d2_small_integers_are_exact(oracle):
    # sum of squares of small integers is exact in binary32 in any order
    for d in (4, 8, 128, 132, 960):
        x = (np.arange(d) % 7).astype(np.float32)
        q = np.zeros(d, np.float32)
        assert oracle.exact_d2(q, x) == np.float32(((np.arange(d) % 7) ** 2).sum())
    e = np.zeros(128, np.float32); e[77] = 3.0
    assert oracle.exact_d2(np.zeros(128, np.float32), e) == 9.0
    assert oracle.exact_d2(e, e) == 0.0


def test_exact_d2_matches_float64(oracle, tiny):
    ix, q = tiny.index, tiny.queries
    rng = np.random.default_rng(7)
    qrow = rng.integers(0, q.shape[0], 500)
    pos = rng.integers(0, ix.n, 500)
    got = oracle.exact_pairs(ix.base, q, qrow, pos)
    ref = ((q[qrow].astype(np.float64) - ix.base[pos].astype(np.float64)) ** 2).sum(1)
    np.testing.assert_allclose(got, ref, rtol=2e-6)
    # symmetric in its arguments (a transposed operand cannot hide)
    assert oracle.exact_d2(q[0], ix.base[5]) == oracle.exact_d2(ix.base[5], q[0])


def test_exact_d2_every_coordinate_counts(oracle):
    # a dropped or doubly-counted coordinate changes one of these
    for d in (128, 960, 1536):
        for t in (0, 3, 4, 127, d - 1, d // 2 + 1):
            x = np.zeros(d, np.float32); x[t] = 2.0
            assert oracle.exact_d2(np.zeros(d, np.float32), x) == 4.0


# ---- the distance table and Gamma(l,q)^2 (Section 3.1: "exactly computed") ------------

def test_table_sum_is_distance_to_reconstruction(oracle, tiny, tiny_ivf):
    for b in (tiny, tiny_ivf):
        ix, q = b.index, b.queries
        lut = oracle.build_lut(q, ix.codebooks)
        rng = np.random.default_rng(3)
        qrow = rng.integers(0, q.shape[0], 400)
        pos = rng.integers(0, ix.n, 400)
        s, _ = oracle.plb_pairs(lut, ix.codes, ix.dlx, qrow, pos, 0.0)
        ref = ((q[qrow].astype(np.float64) - _recon(ix)[pos]) ** 2).sum(1)
        np.testing.assert_allclose(s, ref, rtol=1e-5)


def test_lut_entries(oracle, tiny):
    ix, q = tiny.index, tiny.queries
    lut = oracle.build_lut(q[:3], ix.codebooks)
    dsub = ix.d // ix.M
    qs = q[:3].astype(np.float64).reshape(3, ix.M, 1, dsub)
    ref = ((qs - ix.codebooks.astype(np.float64)[None]) ** 2).sum(-1)
    np.testing.assert_allclose(lut, ref, rtol=1e-5, atol=1e-6)


# ---- encode (Section 3.3 step 1) ---------------------------------------------------------

def test_encode_is_argmin_and_dlx_is_landmark_distance(oracle, tiny, tiny_ivf):
    for b in (tiny, tiny_ivf):
        ix = b.index
        dsub = ix.d // ix.M
        x = ix.base.astype(np.float64).reshape(ix.n, ix.M, 1, dsub)
        cb = ix.codebooks.astype(np.float64)[None]
        bad = 0
        for lo in range(0, ix.n, 500):
            dist = ((x[lo:lo + 500] - cb) ** 2).sum(-1)        # [rows][M][256]
            arg = dist.argmin(-1)
            diff = arg != ix.codes[lo:lo + 500]
            if diff.any():
                # only a float32-level near-tie may differ from the float64 argmin
                r, j = np.nonzero(diff)
                got = dist[r, j, ix.codes[lo:lo + 500][r, j]]
                best = dist[r, j, arg[r, j]]
                assert np.all(got - best <= 1e-5 * best)
                bad += diff.sum()
        assert bad <= 2
        ref = np.sqrt(((ix.base.astype(np.float64) - _recon(ix)) ** 2).sum(1))
        np.testing.assert_allclose(ix.dlx, ref, rtol=1e-5)


def test_encode_ties_take_smallest_index(oracle):
    cb = np.zeros((2, 256, 4), np.float32)
    cb[0, :, 0] = 5.0                      # all centroids equal in subspace 0
    cb[1, :, 0] = np.arange(256)[::-1]     # subspace 1: centroid c at 255-c
    x = np.zeros((1, 8), np.float32); x[0, 4] = 200.5   # equidistant from 200 and 201
    codes, dlx = oracle.encode(x, cb)
    assert codes[0, 0] == 0
    assert codes[0, 1] == 54               # values 201 (c=54) and 200 (c=55): smaller index
    assert dlx[0] == np.float32(np.sqrt(np.float32(25.0 + 0.25)))


# ---- the bound: Definitions 1-2, Equations 3-4, Lemma 1 -------------------------------------

def test_hand_worked_triangle(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "triangle_3_4_12.txt"))
            if l.strip() and not l.startswith("#")]
    cb = np.zeros((1, 256, 4), np.float32)
    cb[0, :, 0] = 10.0 * np.arange(256)
    x = np.array([[3, 4, 0, 0]], np.float32)
    q = np.array([[0, 0, 12, 0]], np.float32)
    codes, dlx = oracle.encode(x, cb)
    assert codes[0, 0] == 0 and dlx[0] == 5.0
    lut = oracle.build_lut(q, cb)
    assert lut[0, 0, 0] == 144.0 and lut[0, 0, 1] == 244.0
    z = np.zeros(1, np.int64)
    for gam, want in rows:
        s, g = oracle.plb_pairs(lut, codes, dlx, z, z, float(gam))
        assert s[0] == 144.0 and g[0] == np.float32(want)
    assert oracle.exact_d2(q[0], x[0]) == 169.0


def _pairs(oracle, b, npairs, seed):
    ix, q = b.index, b.queries
    rng = np.random.default_rng(seed)
    qrow = rng.integers(0, q.shape[0], npairs)
    pos = rng.integers(0, ix.n, npairs)
    lut = oracle.build_lut(q, ix.codebooks)
    l64 = _recon(ix)[pos]
    x64 = ix.base[pos].astype(np.float64)
    q64 = q[qrow].astype(np.float64)
    a = np.sqrt(((q64 - l64) ** 2).sum(1))
    bb = np.sqrt(((x64 - l64) ** 2).sum(1))
    d2 = ((q64 - x64) ** 2).sum(1)
    cos = ((x64 - l64) * (q64 - l64)).sum(1) / (a * bb)
    return lut, qrow, pos, a, bb, d2, cos


def test_strict_bound_never_exceeds_true_distance(oracle, tiny, tiny_ivf):
    # Definition 1 with f = (Gamma(l,q) - Gamma(l,x))^2, i.e. gamma = 0
    for b in (tiny, tiny_ivf):
        lut, qrow, pos, a, bb, d2, _ = _pairs(oracle, b, 4000, 11)
        _, g = oracle.plb_pairs(lut, b.index.codes, b.index.dlx, qrow, pos, 0.0)
        assert np.all(g.astype(np.float64) <= d2 * (1 + 1e-5) + 1e-6)
        np.testing.assert_allclose(g, (a - bb) ** 2, rtol=1e-3, atol=1e-3 * d2.mean())


def test_cosine_theorem_pins_the_relaxation_term(oracle, tiny, tiny_ivf):
    # Equation 4 rearranged: with gamma = 1 - cos(theta) the bound IS Gamma(q,x)^2.
    # A wrong factor (gamma instead of 2*gamma), sign, or a squared b would fail here.
    for b in (tiny, tiny_ivf):
        lut, qrow, pos, a, bb, d2, cos = _pairs(oracle, b, 300, 5)
        ix = b.index
        for i in range(300):
            s, _ = oracle.plb_pairs(lut, ix.codes, ix.dlx, qrow[i:i + 1], pos[i:i + 1], 0.0)
            g = oracle.plb_from_s(s[0], ix.dlx[pos[i]], np.float32(1.0 - cos[i]))
            assert abs(float(g) - d2[i]) <= 2e-4 * d2[i]


def test_two_printed_forms_agree_and_monotone(oracle, tiny):
    # Equation 3 vs the form printed in Section 4.2: a^2 + b^2 - 2ab(1-gamma)
    lut, qrow, pos, a, bb, d2, _ = _pairs(oracle, tiny, 1000, 9)
    ix = tiny.index
    prev = None
    for gam in (0.0, 0.3, 0.7, 1.0):
        _, g = oracle.plb_pairs(lut, ix.codes, ix.dlx, qrow, pos, gam)
        ref = a * a + bb * bb - 2 * a * bb * (1 - gam)
        np.testing.assert_allclose(g, ref, rtol=1e-4, atol=1e-4 * (a * a).mean())
        if prev is not None:
            assert np.all(g >= prev)       # "adding a positive term"
        prev = g


def test_bound_special_cases(oracle):
    # Gamma(l,x) = 0 gives the plain PQ estimate s; gamma = 1 gives a^2 + b^2 (Section 4.2)
    for s in (0.0, 1.0, 144.0, 12345.678):
        assert oracle.plb_from_s(s, 0.0, 0.7) == np.float32(np.float32(np.sqrt(np.float32(s))) ** 2)
    assert oracle.plb_from_s(144.0, 5.0, 1.0) == 169.0
    assert oracle.plb_from_s(0.0, 3.0, 0.5) == 9.0
    assert oracle.plb_from_s(25.0, 5.0, 0.0) == 0.0


# ---- kNN / range by definition (Section 2.1) and the scan (Section 4.2) ---------------------

def _np_brute(b, k):
    """Top-k per query over that query's candidate set, float64, numpy only."""
    ix, out = b.index, []
    for qi in range(b.queries.shape[0]):
        if b.probes is None:
            pos = np.arange(ix.n)
        else:
            pos = np.concatenate([np.arange(ix.list_offsets[l], ix.list_offsets[l + 1])
                                  for l in b.probes[qi]])
        d2 = ((b.queries[qi].astype(np.float64) - ix.base[pos].astype(np.float64)) ** 2).sum(1)
        ids = pos if ix.ids is None else ix.ids[pos]
        o = np.lexsort((ids, d2))[:k]
        out.append((ids[o], d2[o], pos, d2))
    return out


@pytest.mark.parametrize("which", ["tiny", "tiny_ivf"])
def test_strict_knn_equals_brute_force(oracle, which, request):
    b = request.getfixturevalue(which)
    k = 10
    ref = _np_brute(b, k)
    bi, bd = oracle.brute_knn(b.index, b.queries, k, b.probes)
    for batch in (1, 7, 256):
        r = oracle.search_knn(b.index, b.queries, k, 0.0, batch, b.probes)
        np.testing.assert_array_equal(r["ids"], bi)
        np.testing.assert_array_equal(r["d2"], bd)
    for qi, (ids, d2, pos, _) in enumerate(ref):
        np.testing.assert_allclose(bd[qi], d2, rtol=2e-6)
        # ids equal float64's except where two float64 distances are within rounding
        if not np.array_equal(bi[qi], ids):
            assert set(bi[qi]) ^ set(ids) == set() or np.min(np.diff(d2)) < 1e-5 * d2[-1]
        assert r["n_scanned"][qi] == pos.shape[0]
    assert np.all(r["n_exact"] <= r["n_scanned"])
    assert r["n_exact"].sum() < 0.8 * r["n_scanned"].sum()      # it does prune


def test_float64_brute_force_is_the_definition(oracle, tiny, tiny_ivf):
    """brute_knn_f64 (the ground truth behind recall@k, Section 2.1) against numpy's float64
    distances over ALL n, ids through the position -> id map, ties to the smaller id; with
    planted duplicates so that the tie rule is exercised; short inputs are padded."""
    for b in (tiny, tiny_ivf):
        ix, k = b.index, 7
        base = ix.base.copy()
        base[11] = base[3]; base[200] = base[3]            # three equal rows: ties on every query
        ids = ix.ids if ix.ids is not None else np.arange(ix.n, dtype=np.int32)
        got_i, got_d = oracle.brute_knn_f64(base, b.queries, k, ids=ix.ids)
        q64, x64 = b.queries.astype(np.float64), base.astype(np.float64)
        for qi in range(b.queries.shape[0]):
            d2 = ((q64[qi][None, :] - x64) ** 2).sum(1)
            o = np.lexsort((ids, d2))[:k]
            np.testing.assert_array_equal(got_i[qi], ids[o])
            np.testing.assert_allclose(got_d[qi], d2[o], rtol=1e-13)
        # a query equal to the triplicated row: the three copies come first, by ascending id
        gi, gd = oracle.brute_knn_f64(base, np.ascontiguousarray(base[3:4]), 3, ids=ix.ids)
        assert list(gi[0]) == sorted(int(ids[p]) for p in (3, 11, 200)) and np.all(gd == 0.0)
    # fewer than k vectors: padded with (-1, +inf)
    gi, gd = oracle.brute_knn_f64(np.ascontiguousarray(tiny.index.base[:4]), tiny.queries[:2], 6)
    assert np.all(gi[:, 4:] == -1) and np.all(np.isinf(gd[:, 4:])) and np.all(gi[:, :4] >= 0)
    # and it agrees with the binary32 brute force wherever the binary64 distances are well apart
    bi, _ = oracle.brute_knn(tiny.index, tiny.queries, 10)
    fi, fd = oracle.brute_knn_f64(tiny.index.base, tiny.queries, 10)
    for qi in range(tiny.queries.shape[0]):
        if np.min(np.diff(fd[qi])) > 1e-5 * fd[qi][-1]:
            np.testing.assert_array_equal(bi[qi], fi[qi])


@pytest.mark.parametrize("which", ["tiny", "tiny_ivf"])
def test_strict_range_equals_brute_force(oracle, which, request):
    b = request.getfixturevalue(which)
    radius = helpers.radius_at_percentile(b, 1.0, 20, 1000)
    r = oracle.search_range(b.index, b.queries, radius, 0.0, b.probes, want_mask=True)
    r2 = np.float64(np.float32(radius) * np.float32(radius))
    total = 0
    for qi, (_, _, pos, d2) in enumerate(_np_brute(b, 1)):
        ids = pos if b.index.ids is None else b.index.ids[pos]
        got = r["ids"][r["offsets"][qi]:r["offsets"][qi + 1]]
        clear = np.abs(d2 - r2) > 1e-5 * r2          # away from the float32 boundary
        want = ids[(d2 <= r2) & clear]
        assert set(want) <= set(got) <= set(ids[(d2 <= r2) | ~clear])
        # scan order: positions ascending inside the concatenated lists
        order = {int(i): n for n, i in enumerate(ids)}
        seq = [order[int(i)] for i in got]
        assert seq == sorted(seq)
        total += len(got)
    assert total > 0


def test_relaxed_results_are_true_distances_and_nested(oracle, tiny_ivf):
    b = tiny_ivf
    k = 10
    bi, bd = oracle.brute_knn(b.index, b.queries, k, b.probes)
    prev_exact = None
    for gam in (0.0, 0.4, 0.8):
        r = oracle.search_knn(b.index, b.queries, k, gam, 64, b.probes)
        assert np.all(r["d2"] >= bd)                  # i-th returned >= i-th exact
        id2pos = np.empty(b.index.n, np.int64); id2pos[b.index.ids] = np.arange(b.index.n)
        qrow = np.repeat(np.arange(b.queries.shape[0]), k)
        d2 = oracle.exact_pairs(b.index.base, b.queries, qrow, id2pos[r["ids"].ravel()])
        np.testing.assert_array_equal(d2, r["d2"].ravel())
        if prev_exact is not None:
            assert r["n_exact"].sum() <= prev_exact
        prev_exact = r["n_exact"].sum()
    radius = helpers.radius_at_percentile(b, 2.0, 20, 1000)
    prev = None
    for gam in (0.0, 0.4, 0.8):
        r = oracle.search_range(b.index, b.queries, radius, gam, b.probes, want_mask=True)
        sets = [set(r["ids"][r["offsets"][q]:r["offsets"][q + 1]]) for q in range(b.queries.shape[0])]
        if prev is not None:
            assert all(s <= p for s, p in zip(sets, prev[0]))      # results nested
            assert np.all((r["mask"] & ~prev[1]) == 0)              # survivors nested
        prev = (sets, r["mask"])


def test_wrongly_pruned_neighbours_obey_lemma_1(oracle, tiny):
    # a true neighbour can be lost at gamma only if gamma > 1 - cos(theta) for it (Lemma 1)
    b, k, gam = tiny, 10, 0.9
    ix = b.index
    bi, _ = oracle.brute_knn(ix, b.queries, k)
    r = oracle.search_knn(ix, b.queries, k, gam, 32)
    rec = _recon(ix)
    lost = 0
    for qi in range(b.queries.shape[0]):
        for i in set(bi[qi]) - set(r["ids"][qi]):
            l = rec[i]; x = ix.base[i].astype(np.float64); q = b.queries[qi].astype(np.float64)
            cos = ((x - l) * (q - l)).sum() / np.sqrt(((x - l) ** 2).sum() * ((q - l) ** 2).sum())
            assert gam > 1 - cos - 1e-6
            lost += 1
    assert lost > 0        # gamma = 0.9 is aggressive enough to show the effect


def test_batch_one_is_the_sequential_rule(oracle, tiny):
    # Section 4.2 read literally: R = first k vectors; then one vector at a time against maxDis
    b, k, gam = tiny, 5, 0.5
    ix = b.index
    lut = oracle.build_lut(b.queries, ix.codebooks)
    r = oracle.search_knn(ix, b.queries, k, gam, 1, want_mask=True)
    for qi in range(4):
        q = b.queries[qi]
        R = []
        nexact = 0
        for pos in range(ix.n):
            if len(R) >= k:
                s, g = oracle.plb_pairs(lut, ix.codes, ix.dlx, np.array([qi]), np.array([pos]), gam)
                if not g[0] <= R[k - 1][0]:
                    assert not (r["mask"][qi, pos // 32] >> (pos % 32)) & 1
                    continue
            assert (r["mask"][qi, pos // 32] >> (pos % 32)) & 1
            R.append((oracle.exact_d2(q, ix.base[pos]), pos)); R.sort(); R = R[:k]
            nexact += 1
        assert [p for _, p in R] == list(r["ids"][qi])
        assert nexact == r["n_exact"][qi]


def test_short_candidate_lists_are_padded(oracle):
    w = synth.scaled(synth.WORKLOADS["C1"], 300, 3)
    b = helpers.build(w)
    r = oracle.search_knn(b.index, b.queries, 10, 0.0, 16)
    assert np.all(r["ids"] >= 0)
    ix = b.index
    small = type(ix)(ix.base[:4].copy(), ix.codes[:4].copy(), ix.dlx[:4].copy(), ix.codebooks)
    r = oracle.search_knn(small, b.queries, 10, 0.0, 16)
    assert np.all(r["ids"][:, 4:] == -1) and np.all(np.isinf(r["d2"][:, 4:]))
    assert np.all(np.sort(r["ids"][:, :4], axis=1) == np.arange(4))


# ---- index building and candidate generation ---------------------------------------------------

def test_kmeans_objective_never_increases_and_is_deterministic():
    w = synth.scaled(synth.WORKLOADS["C1"], 3000, 1)
    base = synth.base_vectors(w)
    tr, init = synth.kmeans_draws(w, 3000, 32, stream=7)
    c1, obj = index_build.kmeans(base[tr][:, :8].copy(), 32, 8, init)
    c2, _ = index_build.kmeans(base[tr][:, :8].copy(), 32, 8, init)
    assert np.array_equal(c1, c2)
    assert all(obj[i + 1] <= obj[i] * (1 + 1e-12) for i in range(len(obj) - 1))
    assert obj[-1] < obj[0]


def test_fixed_rounding_kmeans(oracle):
    """train_pq_fixed / train_ivf_fixed: one Lloyd step replayed by hand (assignment = argmin of
    float64 distances where no tie is near, mean = exact rational mean), the summation order
    shown on values where it matters, the objective never increasing, empty clusters kept."""
    from fractions import Fraction
    from oracle import index_build
    rng = np.random.default_rng(5)
    # (a) one iteration against exact arithmetic on small integers (every sum is exact)
    train = rng.integers(0, 64, size=(600, 8)).astype(np.float32)
    init = rng.choice(600, 256, replace=False)
    cb = index_build.train_pq_fixed(train, 2, 1, init)
    for j in range(2):
        sub = train[:, 4 * j:4 * j + 4].astype(np.float64)
        c0 = sub[init]
        d2 = ((sub[:, None, :] - c0[None, :, :]) ** 2).sum(-1)     # exact: small integers
        a = d2.argmin(1)                                            # first minimum = smallest index
        for c in range(256):
            rows = np.flatnonzero(a == c)
            if len(rows) == 0:
                np.testing.assert_array_equal(cb[j, c], c0[c].astype(np.float32))
                continue
            for t in range(4):
                mean = Fraction(int(sub[rows, t].sum()), len(rows))
                assert cb[j, c, t] == np.float32(float(mean))       # float64 quotient, rounded once
    # (b) rows are added in ascending row order, in float64
    x = np.array([[1e16], [1.0], [-1e16], [1.0]], dtype=np.float64).astype(np.float32)
    x32 = x.astype(np.float64)
    seq = ((x32[0, 0] + x32[1, 0]) + x32[2, 0]) + x32[3, 0]
    got = index_build._update_fixed(x, np.zeros(4, np.int64), np.zeros((2, 1), np.float32))
    assert got[0, 0] == np.float32(seq / 4.0) and got[1, 0] == 0.0  # cluster 1 is empty: kept
    # (c) Lloyd's invariant with the binary32 assignment rule, PQ and coarse
    w = synth.scaled(synth.WORKLOADS["C2"], 6000, 4, nlist=32, nprobe=4)
    base = synth.base_vectors(w)
    def pq_objective(cb):
        codes, dlx = oracle.encode(base, cb)
        return float((dlx.astype(np.float64) ** 2).mean())
    objs = [pq_objective(index_build.train_pq_fixed(base, 32, it, np.arange(256) * 7)) for it in (0, 1, 2, 4)]
    assert all(b <= a * (1 + 1e-6) for a, b in zip(objs, objs[1:])) and objs[-1] < objs[0]
    cen = [index_build.train_ivf_fixed(base, 32, it, np.arange(32) * 11) for it in (0, 1, 3)]
    def ivf_objective(c):
        a = oracle.ivf_probe(base, c, 1)[:, 0]
        return float(((base.astype(np.float64) - c[a].astype(np.float64)) ** 2).sum(1).mean())
    o = [ivf_objective(c) for c in cen]
    assert o[1] <= o[0] * (1 + 1e-6) and o[2] <= o[1] * (1 + 1e-6) and o[2] < o[0]
    # determinism
    np.testing.assert_array_equal(cen[2], index_build.train_ivf_fixed(base, 32, 3, np.arange(32) * 11))


def test_gamma_estimator_ties_confidence_to_equation_3(oracle, tiny):
    """Section 3.2's lemma: with gamma = gamma_x(p) from the sample, the relaxed bound of
    Equation 3 stays below the true squared distance for exactly m = ceil(p Q) of the Q sampled
    queries (cosine theorem: g <= d^2  <=>  gamma <= 1 - cos(theta)); the global value is the
    smallest gamma_x; p = 1 loses no query of the sample."""
    from oracle import gamma_estimator as ge
    b = tiny
    ix = b.index
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(ix.n, 12, replace=False))
    queries = b.queries
    Q = queries.shape[0]
    lm = ge.landmarks(ix.codes[rows], ix.codebooks)
    for p in (1.0, 0.9, 0.5):
        gamma, gx = ge.estimate_gamma_empirical(ix.base, ix.codes, ix.codebooks, rows, queries, p)
        assert gamma == gx.min()
        m = min(Q, max(1, int(np.ceil(np.float32(p).astype(np.float64) * Q))))
        for i, r in enumerate(rows):
            x = ix.base[r].astype(np.float64)
            a = np.sqrt(((queries.astype(np.float64) - lm[i]) ** 2).sum(1))     # Gamma(l, q)
            bb = np.sqrt(((x - lm[i]) ** 2).sum())                              # Gamma(l, x)
            d2 = ((queries.astype(np.float64) - x) ** 2).sum(1)
            g = (a - bb) ** 2 + 2.0 * gx[i] * a * bb                            # Equation 3
            valid = int((g <= d2 * (1 + 1e-12) + 1e-9).sum())
            assert valid >= m
            # a slightly larger gamma would already lose one more query
            g2 = (a - bb) ** 2 + 2.0 * (gx[i] + 1e-7) * a * bb
            assert int((g2 <= d2 * (1 - 1e-12) - 1e-9).sum()) < m or m == Q and valid == Q
    # closed cases: orthogonal and opposite directions
    l = np.zeros(4); x = np.array([1.0, 0, 0, 0])
    qs = np.array([[0, 2.0, 0, 0], [-3.0, 0, 0, 0], [5.0, 0, 0, 0], [0, 0, 0, 0]])
    np.testing.assert_allclose(ge.one_minus_cos(x, l, qs), [1.0, 2.0, 0.0, 1.0], atol=1e-15)
    assert ge.rank_for_p(1.0, 10) == 0 and ge.rank_for_p(0.9, 1000) == 100 and ge.rank_for_p(0.0, 7) == 6


def test_gamma_for_normal_queries_matches_direct_sampling(oracle):
    """The Z^2 = A/(A+B+C) route with the transform theorem against 1 - Z computed directly
    from d-dimensional standard-normal queries: same distribution (theorems of Section 3.2),
    hence nearly the same gamma_x(p); also pins h1, h2 and the d - 2 terms of C."""
    from oracle import gamma_estimator as ge
    rng = np.random.default_rng(11)
    d = 24
    x = rng.normal(size=d) * 0.7 + 0.3
    l = x + rng.normal(size=d) * 0.25
    qn = rng.normal(size=(60000, d))
    direct = np.sort(ge.one_minus_cos(x, l, qn))
    normals = rng.normal(size=(60000, d))
    h1, h2 = ge.h1_h2(x, l)
    u = x - l
    assert abs(h1 - (u @ l) / np.linalg.norm(u)) < 1e-12 and abs(h1 * h1 + h2 * h2 - l @ l) < 1e-9
    z2 = np.sort(ge.z2_samples(h1, h2, normals))
    y = np.linspace(0.0, 2.0, 401)
    f_route = ge.cdf_one_minus_z_from_z2(z2, y)
    f_direct = np.searchsorted(direct, y, side="right") / direct.shape[0]
    # |Z| has the same law on both sides; the transform theorem itself treats Z as symmetric
    # (its proof halves P(Z^2 >= .)), so the comparison is made on Z^2, and on 1 - Z where that
    # symmetry holds: a landmark at the origin
    z2_direct = np.sort((1.0 - direct) ** 2)
    grid = np.linspace(0, 1, 201)
    ks = np.abs(np.searchsorted(z2, grid) / z2.shape[0] - np.searchsorted(z2_direct, grid) / z2_direct.shape[0]).max()
    assert ks < 0.012
    # one term fewer in C (the text's chi_{d-3}) is visibly different at this sample size
    z2_wrong = np.sort(ge.z2_samples(h1, h2, normals[:, :d - 1]))
    ks_wrong = np.abs(np.searchsorted(z2_wrong, grid) / z2.shape[0] - np.searchsorted(z2_direct, grid) / z2_direct.shape[0]).max()
    assert ks_wrong > 2 * ks
    l0 = np.zeros(d)
    direct0 = np.sort(ge.one_minus_cos(x, l0, qn))
    z20 = np.sort(ge.z2_samples(*ge.h1_h2(x, l0), normals))
    f0 = ge.cdf_one_minus_z_from_z2(z20, y)
    assert np.abs(f0 - np.searchsorted(direct0, y, side="right") / direct0.shape[0]).max() < 0.012
    for p in (0.99, 0.9, 0.6):
        g_route = ge.gamma_normal_queries(x, l0, normals, p)
        g_direct = ge.gamma_from_sample(direct0, p)
        assert abs(g_route - g_direct) < 0.02
    assert f_route[0] <= 0.5 and abs(f_route[-1] - 1.0) < 1e-12


def test_ivf_lists_and_probes(oracle, tiny_ivf):
    b = tiny_ivf
    ix = b.index
    assert sorted(ix.ids.tolist()) == list(range(ix.n))
    for l in range(b.w.nlist):
        seg = ix.ids[ix.list_offsets[l]:ix.list_offsets[l + 1]]
        assert np.all(np.diff(seg) > 0)
    d2 = ((b.queries.astype(np.float64)[:, None, :] - b.centroids.astype(np.float64)[None]) ** 2).sum(-1)
    ref = np.argsort(d2, axis=1, kind="stable")[:, :b.w.nprobe]
    assert np.array_equal(ref, b.probes)
    # every base vector sits in the list of its nearest centroid
    x = ix.base.astype(np.float64)
    a = ((x[:, None, :] - b.centroids.astype(np.float64)[None]) ** 2).sum(-1).argmin(1)
    assert np.array_equal(np.searchsorted(ix.list_offsets, np.arange(ix.n), side="right") - 1, a)


def test_generator_matches_theorem_1_moments():
    # iid N(0, sigma^2) coordinates: E[Gamma^2] = 2 d sigma^2, Var = 8 d sigma^4 (Theorem 1 proof)
    w = synth.Workload("iid", 4000, 4000, 64, 16, 1, "unit")
    r = np.random.default_rng(0)
    x = r.standard_normal((4000, 64)); y = r.standard_normal((4000, 64))
    g2 = ((x - y) ** 2).sum(1)
    assert abs(g2.mean() - 2 * 64) < 2.0 and abs(g2.var() - 8 * 64) < 60
    # the workloads' own laws: value ranges and reproducibility
    for name in ("C1", "C3", "C4"):
        ws = synth.scaled(synth.WORKLOADS[name], 500, 5)
        a, b2 = synth.base_vectors(ws), synth.base_vectors(ws)
        assert np.array_equal(a, b2) and a.dtype == np.float32
        if ws.law == "clip255":
            assert a.min() >= 0 and a.max() <= 255
        elif ws.law == "aniso01":
            assert a.min() >= 0 and a.max() <= 1
        else:
            np.testing.assert_allclose(np.linalg.norm(a, axis=1), 1.0, rtol=1e-5)
