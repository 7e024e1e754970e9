"""GPU parity at the benchmark's full size (C2: 1,000,000 x 128, IVF 1024/32, PQ 32x256,
10,000 queries), in the launch configuration bench.py times.  The oracle cannot process
10^9 (query, candidate) pairs in seconds, so it is run on sampled queries / rows / pairs,
each of which it computes in full; properties that hold at any size are checked on all
outputs."""
import numpy as np
import pytest

from paper_2508_17828_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2(oracle):
    import torch
    from paper_2508_17828_amd import index_setup, trim
    trim.lib()
    w = synth.WORKLOADS["C2"]
    bw = index_setup.build_workload(w)
    ix = bw.index
    h = lambda t: t.cpu().numpy()
    host = oracle.Index(h(ix.base), h(ix.codes), h(ix.dlx), h(ix.codebooks), ids=h(ix.ids),
                        list_offsets=h(ix.list_offsets), centroids=h(bw.centroids))
    probes = trim.trim_ivf_probe(bw.queries, bw.centroids, w.nprobe)
    torch.cuda.synchronize()
    return dict(w=w, bw=bw, host=host, queries=h(bw.queries), probes=probes, trim=trim)


def test_encode_every_row(c2, oracle):
    """The index the other tests hand to the oracle was encoded by the library: all 1,000,000
    codes and landmark distances equal the oracle's own encoding."""
    host = c2["host"]
    codes, dlx = oracle.encode(host.base, host.codebooks)
    np.testing.assert_array_equal(codes, host.codes)
    np.testing.assert_array_equal(dlx.view(np.uint32), host.dlx.view(np.uint32))


def test_strict_scan_of_all_n_is_brute_force(c2, oracle):
    """No candidate structure, gamma = 0, batches of 4096 over all 1,000,000 vectors: the launch
    shape of an exhaustive search.  Ids and distances equal the oracle's brute force."""
    T, w, bw, host = c2["trim"], c2["w"], c2["bw"], c2["host"]
    nq = 200
    r = T.trim_search_knn(bw.index, bw.queries[:nq].contiguous(), w.k, 0.0, 4096)
    bi, bd = oracle.brute_knn(host, np.ascontiguousarray(c2["queries"][:nq]), w.k)
    np.testing.assert_array_equal(r["ids"].cpu().numpy(), bi)
    np.testing.assert_array_equal(r["d2"].cpu().numpy().view(np.uint32), bd.view(np.uint32))
    assert np.all(r["n_scanned"].cpu().numpy() == w.n)
    fi, _ = oracle.brute_knn_f64(host.base, np.ascontiguousarray(c2["queries"][:nq]), w.k, ids=host.ids)
    assert np.mean(fi == bi) > 0.999     # binary64 order differs only at near-ties


def test_probe_selection_sampled_queries(c2, oracle):
    qs = np.sort(synth.sample_indices(77, 1, c2["w"].nq, 300))
    ref = oracle.ivf_probe(np.ascontiguousarray(c2["queries"][qs]), c2["host"].centroids, c2["w"].nprobe)
    np.testing.assert_array_equal(c2["probes"].cpu().numpy()[qs], ref)


@pytest.mark.parametrize("gamma", [0.0, 0.4, 0.8])
def test_knn_full_batch_sampled_against_oracle(c2, oracle, gamma):
    import torch
    T, w, bw, host = c2["trim"], c2["w"], c2["bw"], c2["host"]
    full = T.trim_search_knn(bw.index, bw.queries, w.k, gamma, w.batch, probes=c2["probes"])
    ids = full["ids"].cpu().numpy()
    d2 = full["d2"].cpu().numpy()
    # properties of every row
    assert np.all(np.diff(d2, axis=1) >= 0)
    assert np.all(ids >= 0) and np.all(ids < w.n)
    assert all(len(set(r)) == w.k for r in ids[::97])
    assert np.all(full["n_exact"].cpu().numpy() <= full["n_scanned"].cpu().numpy())
    # sampled queries: the oracle runs each of them in full
    qs = np.sort(synth.sample_indices(78, int(gamma * 10), w.nq, 24))
    hp = c2["probes"].cpu().numpy()[qs]
    hq = np.ascontiguousarray(c2["queries"][qs])
    ref = oracle.search_knn(host, hq, w.k, gamma, w.batch, hp, want_mask=True)
    np.testing.assert_array_equal(ids[qs], ref["ids"])
    np.testing.assert_array_equal(d2[qs], ref["d2"])
    np.testing.assert_array_equal(full["n_exact"].cpu().numpy()[qs], ref["n_exact"])
    np.testing.assert_array_equal(full["n_scanned"].cpu().numpy()[qs], ref["n_scanned"])
    sub = T.trim_search_knn(bw.index, bw.queries[torch.from_numpy(qs).cuda()].contiguous(), w.k,
                            gamma, w.batch, probes=c2["probes"][torch.from_numpy(qs).cuda()].contiguous(),
                            want_mask=True)
    mw = ref["mask"].shape[1]
    np.testing.assert_array_equal(sub["mask"].cpu().numpy().view(np.uint32)[:, :mw], ref["mask"])
    np.testing.assert_array_equal(sub["ids"].cpu().numpy(), ref["ids"])
    # returned distances are the exact distances of the returned ids (sampled pairs)
    id2pos = np.empty(w.n, np.int64); id2pos[host.ids] = np.arange(w.n)
    pr = synth.sample_indices(79, 0, w.nq * w.k, 3000)
    got = oracle.exact_pairs(host.base, c2["queries"], pr // w.k, id2pos[ids.ravel()[pr]])
    np.testing.assert_array_equal(got, d2.ravel()[pr])
    if gamma == 0.0:
        bi, bd = oracle.brute_knn(host, hq, w.k, hp)
        np.testing.assert_array_equal(ids[qs], bi)


@pytest.mark.parametrize("gamma,batch,k", [(0.45, 1024, 10), (0.0, 1024, 10), (0.8, 1024, 10), (0.4, 16, 10),
                                           (0.4, 1, 10), (0.3, 128, 10), (0.45, 1024, 100), (0.4, 16, 100)])
def test_knn_every_query_against_oracle(c2, oracle, gamma, batch, k):
    """All 10,000 queries at the benchmark's operating point: result ids, distances and both
    counters of every query equal the oracle's (the oracle scans them on all host threads; the
    per-candidate masks are compared on the sampled queries above)."""
    T, w, bw, host = c2["trim"], c2["w"], c2["bw"], c2["host"]
    order = T.trim_query_order(c2["probes"], w.nlist)      # as the benchmark launches it
    full = T.trim_search_knn(bw.index, bw.queries, k, gamma, batch, probes=c2["probes"], query_order=order)
    ref = oracle.search_knn(host, c2["queries"], k, gamma, batch, c2["probes"].cpu().numpy())
    np.testing.assert_array_equal(full["ids"].cpu().numpy(), ref["ids"])
    np.testing.assert_array_equal(full["d2"].cpu().numpy().view(np.uint32), ref["d2"].view(np.uint32))
    np.testing.assert_array_equal(full["n_exact"].cpu().numpy(), ref["n_exact"])
    np.testing.assert_array_equal(full["n_scanned"].cpu().numpy(), ref["n_scanned"])


@pytest.mark.parametrize("batch", [1, 16, 100])
def test_knn_small_batches_sampled_against_oracle(c2, oracle, batch):
    """Small batches down to batch = 1, the paper's vector-at-a-time rule, at the benchmark's
    full size (stage B by replay, long barrier-free stretches with bucketed possibles)."""
    T, w, bw, host = c2["trim"], c2["w"], c2["bw"], c2["host"]
    gamma = 0.4
    full = T.trim_search_knn(bw.index, bw.queries, w.k, gamma, batch, probes=c2["probes"], want_mask=True)
    ids, d2 = full["ids"].cpu().numpy(), full["d2"].cpu().numpy()
    assert np.all(np.diff(d2, axis=1) >= 0) and np.all(ids >= 0)
    qs = np.sort(synth.sample_indices(81, batch, w.nq, 16))
    hp = c2["probes"].cpu().numpy()[qs]
    ref = oracle.search_knn(host, np.ascontiguousarray(c2["queries"][qs]), w.k, gamma, batch, hp, want_mask=True)
    np.testing.assert_array_equal(ids[qs], ref["ids"])
    np.testing.assert_array_equal(d2[qs], ref["d2"])
    np.testing.assert_array_equal(full["n_exact"].cpu().numpy()[qs], ref["n_exact"])
    mw = ref["mask"].shape[1]
    np.testing.assert_array_equal(full["mask"].cpu().numpy().view(np.uint32)[qs][:, :mw], ref["mask"])


def test_range_full_batch_sampled_against_oracle(c2, oracle):
    T, w, bw, host = c2["trim"], c2["w"], c2["bw"], c2["host"]
    knn = T.trim_search_knn(bw.index, bw.queries, w.k, 0.0, w.batch, probes=c2["probes"])
    radius = float(np.sqrt(np.median(knn["d2"][:, w.k - 1].cpu().numpy())))
    for gamma in (0.0, 0.5):
        r = T.trim_search_range(bw.index, bw.queries, radius, gamma, probes=c2["probes"])
        off = r["offsets"].cpu().numpy()
        assert off[0] == 0 and np.all(np.diff(off) >= 0) and off[-1] == r["required"]
        assert np.all(r["d2"].cpu().numpy() <= np.float32(radius) * np.float32(radius))
        qs = np.sort(synth.sample_indices(80, 0, w.nq, 16))
        ref = oracle.search_range(host, np.ascontiguousarray(c2["queries"][qs]), radius, gamma,
                                  c2["probes"].cpu().numpy()[qs])
        gi, gd = r["ids"].cpu().numpy(), r["d2"].cpu().numpy()
        ne = r["n_exact"].cpu().numpy()
        for j, q in enumerate(qs):
            np.testing.assert_array_equal(gi[off[q]:off[q + 1]], ref["ids"][ref["offsets"][j]:ref["offsets"][j + 1]])
            np.testing.assert_array_equal(gd[off[q]:off[q + 1]], ref["d2"][ref["offsets"][j]:ref["offsets"][j + 1]])
            assert ne[q] == ref["n_exact"][j]


def test_four_bit_codes_every_query_against_oracle(oracle):
    """C2 indexed with the 4-bit codes of the FastScan variant (64 subspaces of 16 centroids), all
    10,000 queries in the launch configuration bench.py --code-bits 4 times: ids, distances and
    both counters of every query equal oracle/trim_oracle_fs's; the library's encoding of all
    1,000,000 rows equals the oracle's."""
    import torch
    from oracle import trim_oracle_fs as fs
    from paper_2508_17828_amd import index_setup, trim
    w = synth.WORKLOADS["C2"]
    bw = index_setup.build_workload(w, code_bits=4)
    ix = bw.index
    h = lambda t: t.cpu().numpy()
    host = fs.Index(h(ix.base), h(ix.codes), h(ix.dlx), h(ix.codebooks), ids=h(ix.ids),
                    list_offsets=h(ix.list_offsets), centroids=h(bw.centroids))
    codes, dlx = fs.encode(host.base, host.codebooks)
    np.testing.assert_array_equal(codes, host.codes)
    np.testing.assert_array_equal(dlx.view(np.uint32), host.dlx.view(np.uint32))
    probes = trim.trim_ivf_probe(bw.queries, bw.centroids, w.nprobe)
    order = trim.trim_query_order(probes, w.nlist)
    for gamma, batch in ((0.4, 1024), (0.0, 1024), (0.4, 16)):
        full = trim.trim_search_knn(ix, bw.queries, w.k, gamma, batch, probes=probes, query_order=order)
        ref = fs.search_knn(host, h(bw.queries), w.k, gamma, batch, h(probes))
        np.testing.assert_array_equal(full["ids"].cpu().numpy(), ref["ids"])
        np.testing.assert_array_equal(full["d2"].cpu().numpy().view(np.uint32), ref["d2"].view(np.uint32))
        np.testing.assert_array_equal(full["n_exact"].cpu().numpy(), ref["n_exact"])
        np.testing.assert_array_equal(full["n_scanned"].cpu().numpy(), ref["n_scanned"])
