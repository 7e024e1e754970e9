"""GPU parity: every entry point of libtrim, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Bars: PQ codes, landmark distances (they feed the
masks), survivor masks, counters and result ids bit-exact; squared distances within
1e-4 relative (they are in fact produced in the same rounding order, so equality is
asserted first and the tolerance only documents the contract)."""
import numpy as np
import pytest

from paper_2508_17828_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu

RTOL = 1e-4


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2508_17828_amd import trim
    trim.lib()
    return trim


def to_dev(T, b):
    import torch
    ix = b.index
    dev = "cuda:0"
    t = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    gi = T.Index(t(ix.base), t(ix.codes), t(ix.dlx), t(ix.codebooks), ids=t(ix.ids),
                 list_offsets=t(ix.list_offsets),
                 max_list_len=int(np.diff(ix.list_offsets).max()) if ix.list_offsets is not None else 0)
    if ix.codes.shape[1] % 8 == 0:
        gi.scan_head = T.trim_pack_scan_head(gi.codes, gi.dlx)
    if ix.list_offsets is not None:
        gi.list_bounds = T.trim_pack_list_bounds(gi)
    return gi, t(b.queries), t(b.probes)


def u32(t):
    return t.cpu().numpy().view(np.uint32)


CASES = {
    # name: (workload, n, nq, nlist, nprobe)
    "c1": ("C1", 0, 0, -1, -1),                 # the full tiny config: 10k x 128, M=16
    "c2s": ("C2", 60_000, 96, 64, 8),            # M=32, dsub=4, IVF; ragged lists
    "c3s": ("C3", 12_000, 24, -1, -1),           # d=960, M=120 (8-byte code loads), k=100
    "c4s": ("C4", 16_000, 32, 32, 6),            # d=1536, M=192: table in two LDS phases
    "c5s": ("C5", 80_000, 64, 128, 16),          # M=32 with many short lists
    "t384s": ("T384", 60_000, 48, 64, 16),       # d=384, M=48: two 768-thread workgroups per CU
}


def case(name):
    wname, n, nq, nlist, nprobe = CASES[name]
    return helpers.cached(wname, n, nq, nlist, nprobe)


# ---- trim_encode ----------------------------------------------------------------------------

@pytest.mark.parametrize("name", list(CASES))
def test_encode(T, oracle, name):
    b = case(name)
    gi, _, _ = to_dev(T, b)
    codes, dlx = T.trim_encode(gi.base, gi.codebooks)
    np.testing.assert_array_equal(codes.cpu().numpy(), b.index.codes)
    np.testing.assert_array_equal(dlx.cpu().numpy().view(np.uint32), b.index.dlx.view(np.uint32))


def test_encode_generic_subvector_length(T, oracle):
    import torch
    rng = np.random.default_rng(5)
    for d, M, n in ((48, 8, 1000), (24, 12, 515), (128, 4, 300)):   # dsub 6, 2, 32
        base = rng.standard_normal((n, d)).astype(np.float32)
        cb = rng.standard_normal((M, 256, d // M)).astype(np.float32)
        rc, rd = oracle.encode(base, cb)
        codes, dlx = T.trim_encode(torch.from_numpy(base).cuda(), torch.from_numpy(cb).cuda())
        np.testing.assert_array_equal(codes.cpu().numpy(), rc)
        np.testing.assert_array_equal(dlx.cpu().numpy().view(np.uint32), rd.view(np.uint32))


# ---- trim_build_lut --------------------------------------------------------------------------

@pytest.mark.parametrize("name", list(CASES))
def test_build_lut(T, oracle, name):
    b = case(name)
    gi, q, _ = to_dev(T, b)
    lut = T.trim_build_lut(q, gi.codebooks)
    ref = oracle.build_lut(b.queries, b.index.codebooks)
    np.testing.assert_array_equal(lut.cpu().numpy().view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("name", ["c1", "c2s", "c3s", "c4s"])
def test_build_lut_matrix_cores(T, oracle, name):
    # expanded form on the MFMA units: equal to the direct form up to rounding of the
    # cancelling terms, i.e. relative to ||q_j||^2 + ||c||^2 (not to the entry itself)
    b = case(name)
    gi, q, _ = to_dev(T, b)
    lut = T.trim_build_lut(q, gi.codebooks, mfma=True).cpu().numpy()
    ref = oracle.build_lut(b.queries, b.index.codebooks).astype(np.float64)
    M, dsub = b.index.M, b.index.d // b.index.M
    qn = (b.queries.astype(np.float64).reshape(-1, M, dsub) ** 2).sum(-1)          # [nq][M]
    cn = (b.index.codebooks.astype(np.float64) ** 2).sum(-1)                       # [M][256]
    scale = qn[:, :, None] + cn[None, :, :]
    assert np.all(lut >= 0)
    assert np.max(np.abs(lut - ref) / scale) < 2e-6
    # and a strict scan fed with this table still returns the brute-force neighbours except
    # where two candidates are tied to within that rounding
    got = T.trim_search_knn(gi, q, 10, 0.0, 256, probes=to_dev(T, b)[2],
                            lut=T.trim_build_lut(q, gi.codebooks, mfma=True))
    bi, bd = oracle.brute_knn(b.index, b.queries, 10, b.probes)
    assert (got["ids"].cpu().numpy() == bi).mean() > 0.999


# ---- trim_train_pq / trim_train_ivf ------------------------------------------------------------

@pytest.mark.parametrize("wname,ns,M,nlist", [("C2", 5000, 32, 48), ("C1", 3000, 16, 20), ("C3", 1500, 120, 12)])
def test_centroid_training_is_bit_equal_to_the_oracle(T, oracle, wname, ns, M, nlist):
    """Lloyd iterations with fixed roundings: initial rows given, binary32 assignment, float64
    means in row order.  Codebooks and coarse centroids must equal the oracle's bit for bit
    (ragged row count, clusters that run empty, 0 iterations = the initial rows)."""
    import torch
    from oracle import index_build
    w = synth.scaled(synth.WORKLOADS[wname], ns, 4)
    train = synth.base_vectors(w)
    g = torch.from_numpy(train).cuda()
    init = synth.sample_indices(900, 0, ns, 256).astype(np.int32)
    init[5] = init[4]                                   # a duplicate start: one cluster runs empty
    for iters in (0, 3):
        want = index_build.train_pq_fixed(train, M, iters, init)
        got = T.trim_train_pq(g, M, iters, torch.from_numpy(init).cuda()).cpu().numpy()
        np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    init_l = synth.sample_indices(901, 0, ns, nlist).astype(np.int32)
    for iters in (0, 4):
        want = index_build.train_ivf_fixed(train, nlist, iters, init_l)
        got = T.trim_train_ivf(g, nlist, iters, torch.from_numpy(init_l).cuda()).cpu().numpy()
        np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))


# ---- trim_estimate_gamma -----------------------------------------------------------------------

@pytest.mark.parametrize("name", ["c2s", "c3s", "c1"])
def test_gamma_from_confidence_level(T, oracle, name):
    """gamma_x(p) is an order statistic of 1 - cos(theta) over the sampled queries, so an error of
    eps in every value moves it by at most eps: binary32 on the GPU against float64 in the
    oracle must agree to a few 1e-6 (asserted at 2e-5), for every sampled vector and for the
    global minimum; Q is not a power of two and spans several sort tiles."""
    import torch
    from oracle import gamma_estimator as ge
    b = case(name)
    gi, q, _ = to_dev(T, b)
    w = synth.scaled(b.w, b.index.n, 1500)
    queries = synth.query_vectors(w)[:1337]
    rows = np.sort(synth.sample_indices(77, 3, b.index.n, 40)).astype(np.int32)
    gq = torch.from_numpy(queries).cuda()
    for p in (1.0, 0.95, 0.5, 0.0):
        want, want_x = ge.estimate_gamma_empirical(b.index.base, b.index.codes, b.index.codebooks,
                                                   rows, queries, p)
        g, gx = T.trim_estimate_gamma(gi, torch.from_numpy(rows).cuda(), gq, p)
        np.testing.assert_allclose(gx.cpu().numpy(), want_x, atol=2e-5, rtol=0)
        assert abs(float(g.item()) - want) <= 2e-5
    with pytest.raises(T.TrimError):
        T.trim_estimate_gamma(gi, torch.from_numpy(rows).cuda(), gq, 1.5)


def test_gamma_for_normal_queries(T, oracle):
    """The standard-normal route of Section 3.2 (Z^2 = A / (A + B + C) and the transform theorem)
    against oracle/gamma_estimator.gamma_normal_queries on the same variates.  Both sides work
    in binary64 on a grid of 20001 values of y; an order statistic that differs in its last bits
    can move the answer by one grid step (1e-4)."""
    import torch
    from oracle import gamma_estimator as ge
    b = case("c2s")
    gi, _, _ = to_dev(T, b)
    rng = np.random.default_rng(21)
    rows = np.sort(rng.choice(b.index.n, 12, replace=False)).astype(np.int32)
    normals = rng.standard_normal((3000, b.index.d)).astype(np.float32)
    lm = ge.landmarks(b.index.codes[rows], b.index.codebooks)
    for p in (1.0, 0.95, 0.6, 0.3):
        g, gx = T.trim_estimate_gamma_normal(gi, torch.from_numpy(rows).cuda(), torch.from_numpy(normals).cuda(), p)
        ref = np.array([ge.gamma_normal_queries(b.index.base[r], lm[i], normals, p) for i, r in enumerate(rows)])
        np.testing.assert_allclose(gx.cpu().numpy(), ref, atol=1.5e-4, rtol=0)
        assert abs(float(g.item()) - ref.min()) <= 1.5e-4
    with pytest.raises(T.TrimError):
        T.trim_estimate_gamma_normal(gi, torch.from_numpy(rows).cuda(), torch.from_numpy(normals).cuda(), 1.5)


# ---- trim_ivf_probe ----------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["c2s", "c4s", "c5s"])
def test_ivf_probe(T, oracle, name):
    import torch
    b = case(name)
    _, q, _ = to_dev(T, b)
    cen = torch.from_numpy(b.centroids).cuda()
    for nprobe in (1, b.w.nprobe, b.w.nlist):
        got = T.trim_ivf_probe(q, cen, nprobe).cpu().numpy()
        np.testing.assert_array_equal(got, oracle.ivf_probe(b.queries, b.centroids, nprobe))


@pytest.mark.parametrize("nlist,d,nq", [(1000, 128, 9), (4093, 20, 7), (4096, 384, 6), (9000, 8, 5),
                                        (37, 516, 5), (8, 4, 3), (1, 12, 2)])
def test_ivf_probe_shapes(T, oracle, nlist, d, nq):
    """Every instance of the probe kernel (4, 2 and 1 queries per workgroup, chosen by the list
    count), list counts that are not a multiple of the 8 rows a half wave takes per pass, vectors
    shorter and longer than the 128 values a half wave holds in registers."""
    import torch
    rng = np.random.default_rng([77, nlist, d])
    cen = rng.normal(size=(nlist, d)).astype(np.float32)
    cen[nlist // 2] = cen[0]                              # equal distances: the smaller list id first
    q = rng.normal(size=(nq, d)).astype(np.float32)
    q[0] = cen[nlist - 1]                                 # a query on a centroid (the last row)
    for nprobe in sorted({1, min(32, nlist), min(64, nlist), min(100, nlist)}):
        got = T.trim_ivf_probe(torch.from_numpy(q).cuda(), torch.from_numpy(cen).cuda(), nprobe)
        np.testing.assert_array_equal(got.cpu().numpy(), oracle.ivf_probe(q, cen, nprobe))


# ---- trim_search_knn ---------------------------------------------------------------------------

def test_ivf_probe_keys_crowded_in_few_columns(T, oracle):
    """The short-list selection looks at the smallest key of each of 64 interleaved columns
    first.  Here the nearest centroids all sit in the same few columns (index mod 64), so far
    more than 64 keys lie under its bound and the general selection has to take over; with the
    centroid order reversed the bound is tight.  Both must give the oracle's lists."""
    import torch
    nlist, d = 1024, 8
    i = np.arange(nlist)
    rank = (i % 64) * 16 + i // 64                      # column c holds ranks 16c .. 16c+15
    for r in (rank, nlist - 1 - i):
        cen = np.zeros((nlist, d), dtype=np.float32)
        cen[:, 0] = r.astype(np.float32)
        cen[:, 3] = 0.25 * (i % 3)
        q = np.zeros((9, d), dtype=np.float32)
        q[:, 0] = -1.0 - np.arange(9, dtype=np.float32)
        q[5:, 0] = nlist + 3.0                            # some queries from the far end
        for nprobe in (1, 7, 32, 33, 64, 65):
            got = T.trim_ivf_probe(torch.from_numpy(q).cuda(), torch.from_numpy(cen).cuda(), nprobe)
            np.testing.assert_array_equal(got.cpu().numpy(), oracle.ivf_probe(q, cen, nprobe))


def check_knn(T, oracle, b, k, gamma, batch, prebuilt_lut=False):
    gi, q, probes = to_dev(T, b)
    lut = T.trim_build_lut(q, gi.codebooks) if prebuilt_lut else None
    got = T.trim_search_knn(gi, q, k, gamma, batch, probes=probes, lut=lut, want_mask=True)
    ref = oracle.search_knn(b.index, b.queries, k, gamma, batch, b.probes, want_mask=True)
    np.testing.assert_array_equal(got["n_scanned"].cpu().numpy(), ref["n_scanned"])
    mw = ref["mask"].shape[1]
    np.testing.assert_array_equal(u32(got["mask"])[:, :mw], ref["mask"])
    np.testing.assert_array_equal(got["n_exact"].cpu().numpy(), ref["n_exact"])
    np.testing.assert_array_equal(got["ids"].cpu().numpy(), ref["ids"])
    np.testing.assert_allclose(got["d2"].cpu().numpy(), ref["d2"], rtol=RTOL)
    np.testing.assert_array_equal(got["d2"].cpu().numpy(), ref["d2"])
    return got, ref


@pytest.mark.parametrize("gamma", [0.0, 0.6])
@pytest.mark.parametrize("batch", [1, 100, 256, 4096])
def test_knn_c1(T, oracle, gamma, batch):
    check_knn(T, oracle, case("c1"), 10, gamma, batch)


@pytest.mark.parametrize("name,k,batch", [("c2s", 10, 1024), ("c2s", 1, 64), ("c2s", 70, 333),
                                          ("c5s", 10, 1024), ("c3s", 100, 4096),
                                          ("c3s", 100, 512), ("c4s", 10, 2048),
                                          ("c3s", 100, 16), ("c2s", 70, 1), ("c2s", 300, 5),
                                          ("t384s", 10, 1024), ("t384s", 64, 96), ("t384s", 3, 1)])
@pytest.mark.parametrize("gamma", [0.0, 0.5, 0.8])
def test_knn_shapes(T, oracle, name, k, batch, gamma):
    got, ref = check_knn(T, oracle, case(name), k, gamma, batch)
    if gamma == 0.0:
        bi, _ = oracle.brute_knn(case(name).index, case(name).queries, k, case(name).probes)
        np.testing.assert_array_equal(got["ids"].cpu().numpy(), bi)


@pytest.mark.parametrize("name", ["c2s", "c4s"])
def test_knn_with_prebuilt_table(T, oracle, name):
    check_knn(T, oracle, case(name), 10, 0.5, 512, prebuilt_lut=True)


def test_knn_large_k(T, oracle):
    check_knn(T, oracle, case("c2s"), 1024, 0.3, 4096)
    check_knn(T, oracle, case("c1"), 200, 0.0, 128)


def test_knn_few_candidates_and_padding(T, oracle):
    import torch
    b = case("c1")
    ix = b.index
    small = type(ix)(ix.base[:7].copy(), ix.codes[:7].copy(), ix.dlx[:7].copy(), ix.codebooks)
    sb = helpers.Built(b.w, small, b.queries[:5].copy(), None, None)
    got, ref = check_knn(T, oracle, sb, 10, 0.0, 16)
    assert np.all(got["ids"].cpu().numpy()[:, 7:] == -1)
    assert np.all(np.isinf(got["d2"].cpu().numpy()[:, 7:]))
    # no queries at all
    gi, q, _ = to_dev(T, sb)
    out = T.trim_search_knn(gi, q[:0], 10, 0.0, 16)
    assert out["ids"].shape == (0, 10)


def test_knn_empty_and_repeated_lists(T, oracle):
    # probes that name empty lists, and the same list twice (scanned twice, as the oracle does)
    b = case("c2s")
    ix = b.index
    lo = ix.list_offsets.copy()
    # empty out list 3 by moving its boundary: lists 3 and 4 become [empty], [3+4]
    lo[4] = lo[3]
    ix2 = type(ix)(ix.base, ix.codes, ix.dlx, ix.codebooks, ids=ix.ids, list_offsets=lo)
    probes = b.probes.copy()
    probes[:, 0] = 3
    probes[:, 2] = probes[:, 1]
    b2 = helpers.Built(b.w, ix2, b.queries, probes, b.centroids)
    check_knn(T, oracle, b2, 10, 0.4, 256)
    probes[:] = 3                                   # nothing to scan at all
    b3 = helpers.Built(b.w, ix2, b.queries, probes, b.centroids)
    got, _ = check_knn(T, oracle, b3, 10, 0.4, 256)
    assert np.all(got["ids"].cpu().numpy() == -1)


def test_knn_long_probe_sequences(T, oracle):
    """2,500 probed lists per query (more segments than the kernel keeps list ids for in
    on-chip memory), short lists, with and without the list summaries."""
    w = synth.scaled(synth.WORKLOADS["C2"], 150_000, 12, nlist=3000, nprobe=2500, kmeans_iters=2)
    b = helpers.build(w, pq_train_max=8192, ivf_train_per_list=16)
    for k, gamma, batch in ((10, 0.4, 1024), (10, 0.0, 16), (100, 0.5, 256)):
        check_knn(T, oracle, b, k, gamma, batch)
    gi, q, probes = to_dev(T, b)
    gi.list_bounds = None
    got = T.trim_search_knn(gi, q, 10, 0.4, 1024, probes=probes, want_mask=True)
    ref = oracle.search_knn(b.index, b.queries, 10, 0.4, 1024, b.probes, want_mask=True)
    np.testing.assert_array_equal(got["ids"].cpu().numpy(), ref["ids"])
    np.testing.assert_array_equal(got["n_exact"].cpu().numpy(), ref["n_exact"])


def test_query_order_changes_nothing_but_scheduling(T, oracle):
    b = case("c5s")
    gi, q, probes = to_dev(T, b)
    order = T.trim_query_order(probes, b.w.nlist)
    o = order.cpu().numpy()
    assert sorted(o.tolist()) == list(range(b.probes.shape[0]))       # a permutation
    assert np.all(np.diff(b.probes[o, 0]) >= 0)                        # grouped by first list
    a = T.trim_search_knn(gi, q, 10, 0.5, 1024, probes=probes, want_mask=True)
    c = T.trim_search_knn(gi, q, 10, 0.5, 1024, probes=probes, want_mask=True, query_order=order)
    for key in ("ids", "d2", "n_exact", "n_scanned", "mask"):
        assert np.array_equal(a[key].cpu().numpy(), c[key].cpu().numpy())
    r = oracle.search_knn(b.index, b.queries, 10, 0.5, 1024, b.probes)
    np.testing.assert_array_equal(c["ids"].cpu().numpy(), r["ids"])
    # an order array with entries outside 0..nq-1: those slots do nothing, the rest is intact
    import torch
    bad = order.clone(); bad[3] = -5; bad[7] = 10 ** 6
    out = (torch.full((q.shape[0], 10), -7, dtype=torch.int32, device="cuda"),
           torch.zeros((q.shape[0], 10), dtype=torch.float32, device="cuda"))
    T.trim_search_knn(gi, q, 10, 0.5, 1024, probes=probes, out=out, query_order=bad)
    got = out[0].cpu().numpy()
    skipped = [int(order[3]), int(order[7])]
    keep = np.setdiff1d(np.arange(q.shape[0]), skipped)
    np.testing.assert_array_equal(got[keep], r["ids"][keep])
    assert np.all(got[skipped] == -7)
    # range searches take the order too; a query it does not name gets no results
    radius = helpers.radius_at_percentile(b, 1.0)
    ra = T.trim_search_range(gi, q, radius, 0.3, probes=probes)
    rb = T.trim_search_range(gi, q, radius, 0.3, probes=probes, query_order=order)
    for key in ("offsets", "ids", "d2", "n_exact"):
        np.testing.assert_array_equal(ra[key].cpu().numpy(), rb[key].cpu().numpy())
    rc = T.trim_search_range(gi, q, radius, 0.3, probes=probes, query_order=bad, want_stats=False)
    ca, cc = np.diff(ra["offsets"].cpu().numpy()), np.diff(rc["offsets"].cpu().numpy())
    np.testing.assert_array_equal(cc[keep], ca[keep])
    assert np.all(cc[skipped] == 0) and ca.sum() > 0


def test_scan_head_is_a_copy_and_changes_no_result(T, oracle):
    """trim_pack_scan_head lays out {code bytes 0..7, dlx} per vector; a search with and
    without it returns the same bits (and both match the oracle).  c2s has candidate counts
    far beyond one batch, so the long barrier-free stretches that use the head are run."""
    import dataclasses
    b = case("c2s")
    gi, q, probes = to_dev(T, b)
    head = gi.scan_head.cpu().numpy()
    want = np.concatenate([b.index.codes[:, :8], b.index.dlx.view(np.uint8).reshape(-1, 4)], axis=1)
    np.testing.assert_array_equal(head, want)
    plain = dataclasses.replace(gi, scan_head=None)
    for gamma, batch in ((0.0, 256), (0.5, 1024)):
        a = T.trim_search_knn(gi, q, 10, gamma, batch, probes=probes, want_mask=True)
        c = T.trim_search_knn(plain, q, 10, gamma, batch, probes=probes, want_mask=True)
        for key in ("ids", "d2", "n_exact", "n_scanned", "mask"):
            assert np.array_equal(a[key].cpu().numpy(), c[key].cpu().numpy()), key
        r = oracle.search_knn(b.index, b.queries, 10, gamma, batch, b.probes)
        np.testing.assert_array_equal(a["ids"].cpu().numpy(), r["ids"])
        np.testing.assert_array_equal(u32(a["d2"]), r["d2"].view(np.uint32))
    import torch
    with pytest.raises(T.TrimError):   # M = 12: the record's 8 code bytes need M % 8 == 0
        T.trim_pack_scan_head(torch.zeros((4, 12), dtype=torch.uint8, device="cuda"),
                              torch.zeros((4,), dtype=torch.float32, device="cuda"))


@pytest.mark.parametrize("name", ["c2s", "c5s", "c4s"])
def test_list_summaries_hold_and_change_no_result(T, oracle, name):
    """The per-list records hold exactly the codes that occur in each list (ascending, padded with
    the first; count 255 beyond 64 distinct codes) and the largest landmark distance; a search
    gives the same masks, counters and results with and without them, equal to the oracle's."""
    from paper_2508_17828_amd import trim as _t
    b = case(name)
    gi, q, probes = to_dev(T, b)
    ix = b.index
    M = ix.codes.shape[1]
    nlist = len(ix.list_offsets) - 1
    rec = gi.list_bounds.cpu().numpy().reshape(nlist, -1)
    boff = (M * 65 + 3) // 4 * 4
    assert rec.shape[1] == (boff + 4 + 15) // 16 * 16
    lo = ix.list_offsets
    for l in range(nlist):
        rows = slice(int(lo[l]), int(lo[l + 1]))
        bmax = rec[l, boff:boff + 4].copy().view(np.float32)[0]
        if lo[l] == lo[l + 1]:
            assert bmax == 0 and not rec[l, M * 64:M * 65].any()
            continue
        assert bmax == ix.dlx[rows].max()
        for j in range(M):
            want = np.unique(ix.codes[rows, j])
            cnt = int(rec[l, M * 64 + j])
            if len(want) > 64:
                assert cnt == 255
                continue
            assert cnt == len(want)
            got = rec[l, j * 64:(j + 1) * 64]
            np.testing.assert_array_equal(got[:cnt], want)
            assert (got[cnt:] == want[0]).all()
    for k, gamma, batch in ((10, 0.3, 256), (100, 0.0, 16), (10, 0.8, 1024)):
        with_b = T.trim_search_knn(gi, q, k, gamma, batch, probes=probes, want_mask=True)
        saved, gi.list_bounds = gi.list_bounds, None
        without = T.trim_search_knn(gi, q, k, gamma, batch, probes=probes, want_mask=True)
        gi.list_bounds = saved
        for key in ("ids", "d2", "n_exact", "n_scanned", "mask"):
            assert np.array_equal(with_b[key].cpu().numpy(), without[key].cpu().numpy()), key
        ref = oracle.search_knn(ix, b.queries, k, gamma, batch, b.probes, want_mask=True)
        np.testing.assert_array_equal(with_b["ids"].cpu().numpy(), ref["ids"])
        mw = ref["mask"].shape[1]
        np.testing.assert_array_equal(u32(with_b["mask"])[:, :mw], ref["mask"])


@pytest.mark.parametrize("name", ["c4s", "c2s"])
def test_tiled_codes_are_a_copy_and_change_no_result(T, oracle, name):
    """trim_pack_codes_tiled regroups the code bytes (blocks of 64 vectors, 16-byte pieces);
    kNN and range searches that read the tiled copy return the same bits as the row-major ones
    and match the oracle."""
    import dataclasses
    b = case(name)
    gi, q, probes = to_dev(T, b)
    codes = b.index.codes
    n, M = codes.shape
    tiled = T.trim_pack_codes_tiled(gi.codes)
    nb = (n + 63) // 64
    padded = np.zeros((nb * 64, M), np.uint8); padded[:n] = codes
    want = padded.reshape(nb, 64, M // 16, 16).transpose(0, 2, 1, 3).reshape(-1)
    np.testing.assert_array_equal(tiled.cpu().numpy(), want)
    gt = dataclasses.replace(gi, codes_tiled=tiled)
    for gamma, batch in ((0.0, 256), (0.5, 1024)):
        a = T.trim_search_knn(gt, q, 10, gamma, batch, probes=probes, want_mask=True)
        c = T.trim_search_knn(gi, q, 10, gamma, batch, probes=probes, want_mask=True)
        for key in ("ids", "d2", "n_exact", "n_scanned", "mask"):
            assert np.array_equal(a[key].cpu().numpy(), c[key].cpu().numpy()), key
        r = oracle.search_knn(b.index, b.queries, 10, gamma, batch, b.probes)
        np.testing.assert_array_equal(a["ids"].cpu().numpy(), r["ids"])
    # k > 64: the kNN instance that reads the tiled copy
    a = T.trim_search_knn(gt, q, 100, 0.5, 512, probes=probes, want_mask=True)
    r = oracle.search_knn(b.index, b.queries, 100, 0.5, 512, b.probes, want_mask=True)
    np.testing.assert_array_equal(a["ids"].cpu().numpy(), r["ids"])
    np.testing.assert_array_equal(a["n_exact"].cpu().numpy(), r["n_exact"])
    np.testing.assert_array_equal(u32(a["mask"])[:, :r["mask"].shape[1]], r["mask"])
    radius = helpers.radius_at_percentile(b, 2.0, 20, 1000)
    a = T.trim_search_range(gt, q, radius, 0.5, probes=probes, want_mask=True)
    r = oracle.search_range(b.index, b.queries, radius, 0.5, b.probes, want_mask=True)
    np.testing.assert_array_equal(a["offsets"].cpu().numpy(), r["offsets"])
    np.testing.assert_array_equal(a["ids"].cpu().numpy(), r["ids"])
    mw = r["mask"].shape[1]
    np.testing.assert_array_equal(u32(a["mask"])[:, :mw], r["mask"])
    import torch
    with pytest.raises(T.TrimError):   # M = 24 is not a whole number of 16-byte pieces
        T.trim_pack_codes_tiled(torch.zeros((4, 24), dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("name,k,batch,gamma", [("c2s", 10, 1024, 0.4), ("c5s", 10, 64, 0.0), ("c3s", 100, 512, 0.3),
                                                ("c4s", 10, 2048, 0.5), ("c1", 10, 256, 0.6)])
def test_work_counters_account_for_every_candidate(T, oracle, name, k, batch, gamma):
    """The optional accounting of a search: results are those of a launch without it, and the
    counters add up: every candidate is a seed, was read in the first pass, or was passed over
    with its list (a stretch that had to be redone is read twice); exact distances computed
    cover the counted survivors; lookups and bytes lie between what the first pass alone and
    a full evaluation of every candidate would need."""
    b = case(name)
    gi, q, probes = to_dev(T, b)
    M = b.index.M
    plain = T.trim_search_knn(gi, q, k, gamma, batch, probes=probes, want_mask=True)
    got = T.trim_search_knn(gi, q, k, gamma, batch, probes=probes, want_mask=True, want_work=True)
    for key in ("ids", "d2", "n_scanned", "n_exact", "mask"):
        np.testing.assert_array_equal(u32(got[key]), u32(plain[key]), err_msg=key)
    w = got["work"].cpu().numpy().astype(np.int64)
    ns, ne = got["n_scanned"].cpu().numpy().astype(np.int64), got["n_exact"].cpu().numpy().astype(np.int64)
    seeds = np.minimum(k, ns)
    first, skipped, cbytes, looks, rows, fullc = (w[:, i] for i in range(6))
    assert np.all(first + skipped + seeds >= ns)
    assert np.all(first + skipped + seeds <= 2 * ns)
    if name in ("c1", "c2s", "c5s"):     # (c3s: the one long stretch overflows its list of possibles and is redone)
        assert np.mean(first + skipped + seeds == ns) > 0.5
    assert np.all(rows >= ne) and np.all(rows <= ns)
    # (a candidate that passes the first 8 subspaces has its sum redone from the start: M + 8 lookups at most)
    assert np.all(fullc <= first) and np.all(looks <= first * (M + 8)) and np.all(looks >= 4 * first)
    assert np.all(cbytes >= 8 * first) and np.all(cbytes <= first * (2 * M + 24) + 64 * 1024 * M)
    assert np.all(w[:, 6:] == 0)
    # range mode: the chunks of a query add up; no list is passed over there
    radius = helpers.radius_at_percentile(b, 2.0)
    r0 = T.trim_search_range(gi, q, radius, gamma, probes=probes)
    r1 = T.trim_search_range(gi, q, radius, gamma, probes=probes, want_work=True)
    for key in ("offsets", "ids", "d2", "n_scanned", "n_exact"):
        np.testing.assert_array_equal(u32(r1[key]) if r1[key].dtype.is_floating_point else r1[key].cpu().numpy(),
                                      u32(r0[key]) if r0[key].dtype.is_floating_point else r0[key].cpu().numpy(), err_msg=key)
    w = r1["work"].cpu().numpy().astype(np.int64)
    np.testing.assert_array_equal(w[:, 0], r1["n_scanned"].cpu().numpy())
    np.testing.assert_array_equal(w[:, 1], 0)
    np.testing.assert_array_equal(w[:, 4], r1["n_exact"].cpu().numpy())
    assert np.all(w[:, 3] <= w[:, 0] * M) and np.all(w[:, 3] >= 4 * w[:, 0])


def test_knn_is_deterministic(T, oracle):
    b = case("c5s")
    gi, q, probes = to_dev(T, b)
    a = T.trim_search_knn(gi, q, 10, 0.7, 1024, probes=probes, want_mask=True)
    c = T.trim_search_knn(gi, q, 10, 0.7, 1024, probes=probes, want_mask=True)
    for key in ("ids", "d2", "n_exact", "mask"):
        assert np.array_equal(a[key].cpu().numpy(), c[key].cpu().numpy())


def test_ceiling_aids_read_what_they_claim(T):
    """The streaming-read aid touches every 16-byte piece exactly once (its checksum is the xor
    of the buffer, ragged tail of under 16 bytes left out); the lookup aid is deterministic."""
    import torch
    rng = np.random.default_rng(7)
    for words, blocks in ((4, 1), (4 * 768 * 512 * 4 + 4 * 37, 768), (1_000_003, 300)):
        host = rng.integers(0, 2**32, size=words, dtype=np.uint32)
        buf = torch.from_numpy(host.view(np.int32)).cuda()
        sink = torch.zeros(blocks, dtype=torch.int32, device="cuda")
        T.trim_ceiling_stream_read(buf, blocks, sink)
        got = np.bitwise_xor.reduce(u32(sink))
        assert got == np.bitwise_xor.reduce(host[: words // 4 * 4])
    a = torch.zeros(64 * 512, dtype=torch.float32, device="cuda")
    c = torch.zeros_like(a)
    T.trim_ceiling_lds_gather(64, 3, 99, a)
    T.trim_ceiling_lds_gather(64, 3, 99, c)
    assert torch.equal(a, c) and bool(torch.isfinite(a).all()) and float(a.min()) >= 0.0
    assert len(torch.unique(a)) > 1000            # lanes follow different code bytes
    for ef in (2, 4):
        T.trim_ceiling_lds_gather(64, 3, 99, a, entry_floats=ef)
        T.trim_ceiling_lds_gather(64, 3, 99, c, entry_floats=ef)
        assert torch.equal(a, c) and bool(torch.isfinite(a).all())
    with pytest.raises(T.TrimError):
        T.trim_ceiling_lds_gather(64, 3, 99, a, entry_floats=3)
    with pytest.raises(T.TrimError):
        T.trim_ceiling_lds_gather(0, 3, 99, a)
    with pytest.raises(T.TrimError):
        T.trim_ceiling_stream_read(buf, 1 << 20, torch.zeros(1 << 20, dtype=torch.int32, device="cuda"))


def test_argument_errors(T):
    import torch
    b = case("c1")
    gi, q, _ = to_dev(T, b)
    for kw in (dict(k=0), dict(k=T.TRIM_MAX_K + 1), dict(batch=0), dict(batch=T.TRIM_MAX_BATCH + 1),
               dict(gamma=-0.1), dict(gamma=float("nan"))):
        args = dict(k=10, gamma=0.0, batch=64); args.update(kw)
        with pytest.raises(T.TrimError):
            T.trim_search_knn(gi, q, args["k"], args["gamma"], args["batch"])
    assert not T.trim_shape_supported(130, 16) and not T.trim_shape_supported(128, 6)
    assert T.trim_shape_supported(128, 32) and T.trim_shape_supported(1536, 192)
    with pytest.raises(TypeError):
        T.trim_encode(gi.base, gi.codebooks[:, :, :7].contiguous())
    with pytest.raises(TypeError):
        T.trim_encode(gi.base.cpu(), gi.codebooks)
    # list summaries: the record size is what the header says; a misaligned buffer, or one that is
    # passed to a search misaligned, is refused
    import ctypes as C
    L = T.lib()
    assert L.trim_list_bounds_bytes(7, 32) == 7 * 2096      # 32 x 64 codes + 32 counts + 4, to 16
    assert L.trim_list_bounds_bytes(0, 32) == 0
    b2 = case("c5s")
    gi2, q2, probes2 = to_dev(T, b2)
    buf = torch.zeros(gi2.list_bounds.numel() + 16, dtype=torch.uint8, device="cuda")
    view = gi2._view()
    nlist = gi2.list_offsets.shape[0] - 1
    assert L.trim_pack_list_bounds(C.byref(view), C.c_void_p(gi2.list_offsets.data_ptr()), nlist,
                                   C.c_void_p(buf.data_ptr() + 4), None) == -1
    assert L.trim_pack_list_bounds(C.byref(view), C.c_void_p(gi2.list_offsets.data_ptr()), 0,
                                   C.c_void_p(buf.data_ptr()), None) == -1
    gi2.list_bounds = buf[4:4 + gi2.list_bounds.numel()]          # a view that starts 4 bytes in
    with pytest.raises(T.TrimError):
        T.trim_search_knn(gi2, q2, 10, 0.0, 64, probes=probes2)


# ---- trim_search_range ---------------------------------------------------------------------------

def check_range(T, oracle, b, radius, gamma):
    gi, q, probes = to_dev(T, b)
    got = T.trim_search_range(gi, q, radius, gamma, probes=probes, want_mask=True)
    ref = oracle.search_range(b.index, b.queries, radius, gamma, b.probes, want_mask=True)
    np.testing.assert_array_equal(got["n_scanned"].cpu().numpy(), ref["n_scanned"])
    mw = ref["mask"].shape[1]
    np.testing.assert_array_equal(u32(got["mask"])[:, :mw], ref["mask"])
    np.testing.assert_array_equal(got["n_exact"].cpu().numpy(), ref["n_exact"])
    np.testing.assert_array_equal(got["offsets"].cpu().numpy(), ref["offsets"])
    np.testing.assert_array_equal(got["ids"].cpu().numpy(), ref["ids"])
    np.testing.assert_allclose(got["d2"].cpu().numpy(), ref["d2"], rtol=RTOL)
    np.testing.assert_array_equal(got["d2"].cpu().numpy(), ref["d2"])
    return got, ref


@pytest.mark.parametrize("name,percent", [("c1", 1.0), ("c2s", 0.5), ("c4s", 0.5), ("c5s", 0.2),
                                          ("c3s", 1.0)])
@pytest.mark.parametrize("gamma", [0.0, 0.7])
def test_range(T, oracle, name, percent, gamma):
    b = case(name)
    radius = helpers.radius_at_percentile(b, percent, 24, 2000)
    got, ref = check_range(T, oracle, b, radius, gamma)
    if gamma == 0.0:
        assert ref["offsets"][-1] > 0


def test_range_degenerate_radii_and_capacity(T, oracle):
    b = case("c2s")
    check_range(T, oracle, b, 0.0, 0.0)                      # nothing within radius 0
    got, ref = check_range(T, oracle, b, 1e6, 0.0)            # everything is a result
    assert ref["offsets"][-1] == ref["n_scanned"].sum()
    gi, q, probes = to_dev(T, b)
    with pytest.raises(T.TrimCapacityError) as e:
        T.trim_search_range(gi, q, 1e6, 0.0, probes=probes, capacity=1000)
    assert e.value.required == ref["offsets"][-1]
    import torch
    with pytest.raises(T.TrimError):
        T.trim_search_range(gi, q, 1.0, 0.0, probes=probes,
                            workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
