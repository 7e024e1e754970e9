"""Pins for the 4-bit-code oracle (oracle/trim_oracle_fs.c; Section 6.1: FastScan variants use
4-bit codes, m = d/2).  As in test_oracle_pins.py, every check compares oracle output with
something fixed outside it: float64 closed forms written here with numpy, brute force by
definition, a hand-made packed code, and the already pinned 8-bit oracle on an index built so
that both must agree.  No GPU is used."""
import numpy as np
import pytest

from oracle import trim_oracle_fs as fs
from tests import helpers


@pytest.fixture(scope="module")
def tiny(oracle):
    return helpers.cached_fs("C1", 2000, 24)            # d=128 -> m=64 subspaces of 2 dims, no lists


@pytest.fixture(scope="module")
def tiny_ivf(oracle):
    return helpers.cached_fs("C2", 6000, 20, 16, 5)     # 16 lists / 5 probes


def _nibbles(codes, m):
    """Own unpacking (not the oracle's): subspace j sits in byte j//2, low half for even j."""
    return np.stack([(codes[:, j // 2] >> (4 * (j % 2))) & 15 for j in range(m)], axis=1)


def _recon(ix):
    m, dsub = ix.m, ix.d // ix.m
    nib = _nibbles(ix.codes, m)
    r = np.empty((ix.n, ix.d), np.float64)
    for j in range(m):
        r[:, j * dsub:(j + 1) * dsub] = ix.codebooks[j][nib[:, j]]
    return r


def test_hand_made_packed_code(oracle):
    """d=8, m=4: table entries chosen so that every subspace's pick is visible in the sum."""
    T = np.zeros((4, 16), np.float32)
    T[0, 3], T[1, 12], T[2, 0], T[3, 15] = 1.0, 10.0, 100.0, 1000.0
    code = np.array([3 | (12 << 4), 0 | (15 << 4)], np.uint8)     # subspaces 0..3 = 3, 12, 0, 15
    assert fs.table_sum(T, code) == 1111.0
    code_swapped = np.array([12 | (3 << 4), 15 | (0 << 4)], np.uint8)
    assert fs.table_sum(T, code_swapped) == 0.0
    # encode puts the even subspace in the low half
    cb = np.zeros((4, 16, 2), np.float32)
    for j in range(4):
        cb[j, :, 0] = np.arange(16) * 10.0
    x = np.array([[30, 0, 120, 0, 0, 0, 150, 0]], np.float32)    # nearest centroids 3, 12, 0, 15
    codes, dlx = fs.encode(x, cb)
    assert list(codes[0]) == [3 | (12 << 4), 0 | (15 << 4)] and dlx[0] == 0.0
    np.testing.assert_array_equal(fs.unpack(codes, 4), [[3, 12, 0, 15]])


def test_table_sum_is_distance_to_reconstruction(oracle, tiny, tiny_ivf):
    """Section 3.1: sum_j T[j][code_j] = || q - landmark ||^2, landmark = PQ reconstruction."""
    for b in (tiny, tiny_ivf):
        ix = b.index
        lut = fs.build_lut(b.queries, ix.codebooks)
        rec = _recon(ix)
        rng = np.random.default_rng(3)
        qrow = rng.integers(0, b.queries.shape[0], 400)
        pos = rng.integers(0, ix.n, 400)
        s, _ = fs.plb_pairs(lut, ix.codes, ix.dlx, qrow, pos, 0.0)
        ref = ((b.queries[qrow].astype(np.float64) - rec[pos]) ** 2).sum(1)
        np.testing.assert_allclose(s, ref, rtol=2e-6)
        # table entries themselves
        j, c, qi = 7, 11, 2
        dsub = ix.d // ix.m
        ref = ((b.queries[qi, j * dsub:(j + 1) * dsub].astype(np.float64) - ix.codebooks[j, c]) ** 2).sum()
        np.testing.assert_allclose(lut[qi, j, c], ref, rtol=1e-6)


def test_encode_is_argmin_and_dlx_is_landmark_distance(oracle, tiny):
    ix = tiny.index
    m, dsub = ix.m, ix.d // ix.m
    nib = _nibbles(ix.codes, m)
    x64 = ix.base.astype(np.float64)
    for j in (0, 1, 17, m - 1):
        dist = ((x64[:, None, j * dsub:(j + 1) * dsub] - ix.codebooks[j][None].astype(np.float64)) ** 2).sum(2)
        best = dist.min(1)
        mine = dist[np.arange(ix.n), nib[:, j]]
        assert np.all(mine <= best * (1 + 1e-6) + 1e-9)
    np.testing.assert_allclose(ix.dlx, np.sqrt(((x64 - _recon(ix)) ** 2).sum(1)), rtol=2e-6)
    assert np.all(ix.codes.shape == (ix.n, m // 2))


def test_encode_ties_take_smallest_index(oracle):
    cb = np.zeros((2, 16, 2), np.float32)
    cb[0, 5:] = 1.0            # centroids 0..4 identical (0,0), 5..15 identical (1,1)
    cb[1, :, 0] = 3.0          # all sixteen identical
    x = np.array([[0, 0, 3, 0], [1, 1, 9, 9]], np.float32)
    codes, _ = fs.encode(x, cb)
    np.testing.assert_array_equal(fs.unpack(codes, 2), [[0, 0], [5, 0]])


def test_strict_bound_never_exceeds_true_distance(oracle, tiny_ivf):
    """Definition 1 with the PQ landmark: g(gamma = 0) <= Gamma(q,x)^2, checked in float64 with the
    binary32 slack of the computed chain."""
    b = tiny_ivf
    ix = b.index
    lut = fs.build_lut(b.queries, ix.codebooks)
    rng = np.random.default_rng(5)
    qrow, pos = rng.integers(0, b.queries.shape[0], 3000), rng.integers(0, ix.n, 3000)
    _, g = fs.plb_pairs(lut, ix.codes, ix.dlx, qrow, pos, 0.0)
    d2 = ((b.queries[qrow].astype(np.float64) - ix.base[pos].astype(np.float64)) ** 2).sum(1)
    assert np.all(g <= d2 * (1 + 1e-5) + 1e-3)
    # and the relaxation adds exactly 2 gamma a b (Equation 3), a and b from float64
    a = np.sqrt(((b.queries[qrow].astype(np.float64) - _recon(ix)[pos]) ** 2).sum(1))
    _, g7 = fs.plb_pairs(lut, ix.codes, ix.dlx, qrow, pos, 0.7)
    np.testing.assert_allclose(g7 - g, 2 * 0.7 * a * ix.dlx[pos].astype(np.float64), rtol=1e-4, atol=1e-2)


def _np_brute(b, k):
    ix, out = b.index, []
    for qi in range(b.queries.shape[0]):
        pos = np.arange(ix.n) if b.probes is None else np.concatenate(
            [np.arange(ix.list_offsets[l], ix.list_offsets[l + 1]) for l in b.probes[qi]])
        d2 = ((b.queries[qi].astype(np.float64) - ix.base[pos].astype(np.float64)) ** 2).sum(1)
        ids = pos if ix.ids is None else ix.ids[pos]
        o = np.lexsort((ids, d2))[:k]
        out.append((ids[o], d2[o], pos, d2))
    return out


@pytest.mark.parametrize("which", ["tiny", "tiny_ivf"])
def test_strict_scan_equals_brute_force(oracle, which, request):
    """gamma = 0: kNN and range results are the definitions of Section 2.1 over the candidates."""
    b = request.getfixturevalue(which)
    k = 10
    ref = _np_brute(b, k)
    for batch in (1, 7, 256):
        r = fs.search_knn(b.index, b.queries, k, 0.0, batch, b.probes)
        for qi, (ids, d2, pos, _) in enumerate(ref):
            np.testing.assert_allclose(r["d2"][qi], d2, rtol=2e-6)
            if not np.array_equal(r["ids"][qi], ids):
                assert np.min(np.diff(d2)) < 1e-5 * d2[-1]
            assert r["n_scanned"][qi] == pos.shape[0]
    assert r["n_exact"].sum() < 0.9 * r["n_scanned"].sum()      # it does prune
    radius = helpers.radius_at_percentile(b, 2.0, 20, 1000)
    rr = fs.search_range(b.index, b.queries, radius, 0.0, b.probes)
    r2 = float(np.float32(radius) * np.float32(radius))
    for qi, (_, _, pos, d2) in enumerate(ref):
        ids = pos if b.index.ids is None else b.index.ids[pos]
        got = rr["ids"][rr["offsets"][qi]:rr["offsets"][qi + 1]]
        sure = ids[d2 <= r2 * (1 - 1e-5)]
        maybe = ids[d2 <= r2 * (1 + 1e-5)]
        assert set(sure) <= set(got) <= set(maybe)
        assert list(got) == [i for i in ids if i in set(got)]     # scan order


def test_batch_one_is_the_sequential_rule(oracle, tiny):
    """B = 1 is the rule of Section 4.2 taken vector by vector: replayed here from the bound and
    the exact distance of each candidate alone."""
    b, k, gam = tiny, 5, 0.5
    ix = b.index
    lut = fs.build_lut(b.queries, ix.codebooks)
    r = fs.search_knn(ix, b.queries, k, gam, 1, want_mask=True)
    for qi in range(4):
        q = b.queries[qi]
        R, nexact = [], 0
        _, g = fs.plb_pairs(lut, ix.codes, ix.dlx, np.full(ix.n, qi), np.arange(ix.n), gam)
        for pos in range(ix.n):
            if pos >= k and not g[pos] <= R[k - 1][0]:
                assert not (r["mask"][qi, pos // 32] >> (pos % 32)) & 1
                continue
            assert (r["mask"][qi, pos // 32] >> (pos % 32)) & 1
            R.append((oracle.exact_d2(q, ix.base[pos]), pos)); R.sort(); R = R[:k]
            nexact += 1
        assert [p for _, p in R] == list(r["ids"][qi])
        assert nexact == r["n_exact"][qi]


def test_relaxed_results_are_nested_and_true(oracle, tiny_ivf):
    b = tiny_ivf
    radius = helpers.radius_at_percentile(b, 2.0, 20, 1000)
    prev = None
    for gam in (0.0, 0.4, 0.8):
        r = fs.search_range(b.index, b.queries, radius, gam, b.probes, want_mask=True)
        if prev is not None:
            assert np.all((r["mask"] & ~prev) == 0)      # survivors(gamma2) within survivors(gamma1)
        prev = r["mask"]
        assert np.all(r["d2"] <= np.float32(radius) * np.float32(radius))


def test_agrees_with_the_eight_bit_oracle_on_a_product_codebook(oracle, tiny):
    """Two neighbouring 16-centroid subspaces are one 256-centroid subspace whose centroid
    (lo | hi << 4) is the concatenation of the two: on that codebook the pinned 8-bit oracle must
    produce the packed codes as its codes, the same landmark distances and table sums up to
    rounding, and the same strict results."""
    b = tiny
    ix = b.index
    m, dsub = ix.m, ix.d // ix.m
    M = m // 2
    cb8 = np.empty((M, 256, 2 * dsub), np.float32)
    for i in range(M):
        for c in range(256):
            cb8[i, c, :dsub] = ix.codebooks[2 * i, c & 15]
            cb8[i, c, dsub:] = ix.codebooks[2 * i + 1, c >> 4]
    codes8, dlx8 = oracle.encode(ix.base, cb8)
    same = codes8 == ix.codes
    assert same.mean() > 0.999                      # (an exact tie may be broken differently)
    np.testing.assert_allclose(dlx8, ix.dlx, rtol=2e-6)
    lut8 = oracle.build_lut(b.queries, cb8)
    lut4 = fs.build_lut(b.queries, ix.codebooks)
    rng = np.random.default_rng(9)
    qrow, pos = rng.integers(0, b.queries.shape[0], 2000), rng.integers(0, ix.n, 2000)
    s8, g8 = oracle.plb_pairs(lut8, ix.codes, ix.dlx, qrow, pos, 0.6)
    s4, g4 = fs.plb_pairs(lut4, ix.codes, ix.dlx, qrow, pos, 0.6)
    np.testing.assert_allclose(s4, s8, rtol=2e-6)
    np.testing.assert_allclose(g4, g8, rtol=1e-4, atol=1e-2)
    ix8 = oracle.Index(ix.base, ix.codes, ix.dlx, cb8)
    np.testing.assert_array_equal(fs.search_knn(ix, b.queries, 10, 0.0, 64)["ids"],
                                  oracle.search_knn(ix8, b.queries, 10, 0.0, 64)["ids"])


def test_fixed_rounding_training_is_lloyd(oracle, tiny):
    """train_pq_fs_fixed: every iteration is an assignment to the nearest of 16 centroids followed by
    the mean of the members; pinned on small integers, where every float64 sum is exact."""
    from oracle import index_build
    rng = np.random.default_rng(11)
    train = rng.integers(0, 9, size=(300, 8)).astype(np.float32)
    init = np.arange(16)
    cb0 = index_build.train_pq_fs_fixed(train, 4, 0, init)
    np.testing.assert_array_equal(cb0, train[init].reshape(16, 4, 2).transpose(1, 0, 2))
    cb1 = index_build.train_pq_fs_fixed(train, 4, 1, init)
    for j in range(4):
        xs = train[:, 2 * j:2 * j + 2].astype(np.float64)
        dist = ((xs[:, None, :] - cb0[j][None].astype(np.float64)) ** 2).sum(2)
        a = dist.argmin(1)                                    # integers: exact, smallest index on ties
        for c in range(16):
            if np.any(a == c):
                np.testing.assert_array_equal(cb1[j, c], xs[a == c].mean(0).astype(np.float32))
            else:
                np.testing.assert_array_equal(cb1[j, c], cb0[j, c])
