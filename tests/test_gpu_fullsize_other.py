"""GPU parity at the full base-set sizes of the remaining workloads: C3 (1M x 960, M=120,
all n scanned, k=100), C4 (1M x 1536, M=192: table in two LDS phases, IVF 1024/64, range
search) and C5 (10M x 128, IVF 4096/64, kNN and range).  The base set, index shape and
launch configuration are the full ones; the query set is cut to 256 queries to bound the
run time, and the oracle, which cannot scan 10^8..10^9 pairs in seconds, is run in full on a
few sampled queries."""
import numpy as np
import pytest

from paper_2508_17828_amd import synth

pytestmark = pytest.mark.gpu

NQ = 256


def build(name, oracle):
    import torch
    from paper_2508_17828_amd import index_setup, trim
    trim.lib()
    w = synth.scaled(synth.WORKLOADS[name], synth.WORKLOADS[name].n, NQ)
    bw = index_setup.build_workload(w)
    ix = bw.index
    h = lambda t: None if t is None else t.cpu().numpy()
    host = oracle.Index(h(ix.base), h(ix.codes), h(ix.dlx), h(ix.codebooks), ids=h(ix.ids),
                        list_offsets=h(ix.list_offsets), centroids=h(bw.centroids))
    probes = trim.trim_ivf_probe(bw.queries, bw.centroids, w.nprobe) if w.nlist else None
    torch.cuda.synchronize()
    return w, bw, host, h(bw.queries), probes, trim


def check_encode_rows(oracle, host, seed):
    rows = np.sort(synth.sample_indices(seed, 0, host.n, 1500))
    codes, dlx = oracle.encode(np.ascontiguousarray(host.base[rows]), host.codebooks)
    np.testing.assert_array_equal(codes, host.codes[rows])
    np.testing.assert_array_equal(dlx.view(np.uint32), host.dlx[rows].view(np.uint32))


def check_knn(oracle, w, bw, host, queries, probes, trim, gamma, nsample, seed):
    full = trim.trim_search_knn(bw.index, bw.queries, w.k, gamma, w.batch, probes=probes)
    ids, d2 = full["ids"].cpu().numpy(), full["d2"].cpu().numpy()
    assert np.all(np.diff(d2, axis=1) >= 0) and np.all(ids >= 0) and np.all(ids < w.n)
    qs = np.sort(synth.sample_indices(seed, 1, NQ, nsample))
    hp = None if probes is None else probes.cpu().numpy()[qs]
    ref = oracle.search_knn(host, np.ascontiguousarray(queries[qs]), w.k, gamma, w.batch, hp)
    np.testing.assert_array_equal(ids[qs], ref["ids"])
    np.testing.assert_array_equal(d2[qs], ref["d2"])
    np.testing.assert_array_equal(full["n_exact"].cpu().numpy()[qs], ref["n_exact"])
    np.testing.assert_array_equal(full["n_scanned"].cpu().numpy()[qs], ref["n_scanned"])


def check_range(oracle, w, bw, host, queries, probes, trim, radius, gamma, nsample, seed):
    r = trim.trim_search_range(bw.index, bw.queries, radius, gamma, probes=probes)
    off, gi, gd = r["offsets"].cpu().numpy(), r["ids"].cpu().numpy(), r["d2"].cpu().numpy()
    assert off[0] == 0 and np.all(np.diff(off) >= 0) and off[-1] == r["required"]
    assert np.all(gd <= np.float32(radius) * np.float32(radius))
    qs = np.sort(synth.sample_indices(seed, 2, NQ, nsample))
    hp = None if probes is None else probes.cpu().numpy()[qs]
    ref = oracle.search_range(host, np.ascontiguousarray(queries[qs]), radius, gamma, hp)
    ne = r["n_exact"].cpu().numpy()
    for j, q in enumerate(qs):
        np.testing.assert_array_equal(gi[off[q]:off[q + 1]], ref["ids"][ref["offsets"][j]:ref["offsets"][j + 1]])
        np.testing.assert_array_equal(gd[off[q]:off[q + 1]], ref["d2"][ref["offsets"][j]:ref["offsets"][j + 1]])
        assert ne[q] == ref["n_exact"][j]
    return int(off[-1])


def radius_from_pairs(w, host, queries, percent):
    qi, bi = synth.pair_sample(w, 64, 10_000)
    q = queries[qi].astype(np.float64)
    x = host.base[np.sort(bi)].astype(np.float64)
    d2 = ((q * q).sum(1)[:, None] - 2 * q @ x.T + (x * x).sum(1)[None, :]).ravel()
    return float(np.sqrt(max(np.percentile(d2, percent), 0.0)))


def test_c3_full_base(oracle):
    w, bw, host, queries, probes, trim = build("C3", oracle)
    check_encode_rows(oracle, host, 91)
    for gamma in w.gammas:
        check_knn(oracle, w, bw, host, queries, probes, trim, gamma, 24, 92)


def test_c4_full_base_range(oracle):
    w, bw, host, queries, probes, trim = build("C4", oracle)
    check_encode_rows(oracle, host, 93)
    radius = radius_from_pairs(w, host, queries, w.range_percentile)
    total = 0
    for gamma in w.gammas:
        total += check_range(oracle, w, bw, host, queries, probes, trim, radius, gamma, 24, 94)
    assert total > 0
    check_knn(oracle, w, bw, host, queries, probes, trim, 0.0, 24, 95)


def test_c5_full_base(oracle):
    w, bw, host, queries, probes, trim = build("C5", oracle)
    check_encode_rows(oracle, host, 96)
    for gamma in (0.0, 0.5):
        check_knn(oracle, w, bw, host, queries, probes, trim, gamma, NQ, 97)   # every query
    radius = radius_from_pairs(w, host, queries, w.range_percentile)
    check_range(oracle, w, bw, host, queries, probes, trim, radius, 0.5, 6, 98)
