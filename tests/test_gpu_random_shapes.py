"""GPU parity on seeded random configurations: dimensions, subspace counts, result sizes,
batch schedules, candidate structures and relaxation drawn at random (within the library's
limits), each checked bit for bit against the oracle for kNN and for range search.  The
fixed cases elsewhere aim at known corners; these walk the plan space (table phases, block
sizes, residency tiers, code-load widths, growing batches, tiled codes, scan head)."""
import numpy as np
import pytest

from paper_2508_17828_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu

LAWS = {"clip255": "C2", "aniso01": "C3", "unit": "C4"}


def draw(seed):
    r = np.random.default_rng([2024, seed])
    M = int(r.choice([4, 8, 12, 16, 24, 32, 48, 64, 96, 120, 160, 192]))
    dsub = int(r.choice([4, 8] if M > 64 else [4, 8, 16]))
    law = str(r.choice(list(LAWS)))
    n = int(r.integers(700, 9000))
    nq = int(r.integers(3, 20))
    use_ivf = bool(r.integers(0, 2))
    nlist = int(r.integers(4, 40)) if use_ivf else 0
    nprobe = int(r.integers(1, nlist + 1)) if use_ivf else 0
    k = int(r.choice([1, 3, 10, 64, 65, 100, 200, 300]))
    batch = int(r.choice([1, 7, 64, 100, 256, 1000, 1024, 2048, 4096]))
    first = int(r.choice([0, 0, 1, 5, 64, batch])) if batch > 1 else 0
    first = min(first, batch)
    gamma = float(r.choice([0.0, 0.3, 0.6, 0.9]))
    base = synth.WORKLOADS[LAWS[law]]
    w = synth.scaled(base, n, nq, d=M * dsub, M=M, nlist=nlist, nprobe=nprobe, k=k,
                     ncomp=int(r.integers(4, 40)), seed=1000 + seed, kmeans_iters=3)
    return w, k, batch, first, gamma


def draw_long(seed):
    """Long candidate lists: several barrier-free stretches per query, ring queues, possibles
    lists that overflow at loose thresholds."""
    r = np.random.default_rng([2025, seed])
    M = int(r.choice([16, 32, 64]))
    dsub = int(r.choice([4, 8]))
    n = int(r.integers(90_000, 260_000))
    k = int(r.choice([10, 64, 100]))
    batch = int(r.choice([128, 256, 1024, 2048]))
    if seed >= 6:      # small batches down to the vector-at-a-time rule: replay, buckets, short spans
        k = int(r.choice([1, 10, 37, 64]))
        batch = int(r.choice([1, 2, 3, 16, 48, 100]))
    if seed >= 14:     # the same with result sets wider than 64 (more than one entry per lane)
        k = int(r.choice([65, 100, 128, 200, 300, 1024]))
        batch = int(r.choice([1, 3, 16, 100, 300]))
    first = int(r.choice([0, 32, batch]))
    first = min(first, batch)
    gamma = float(r.choice([0.0, 0.4, 0.8]))
    law = str(r.choice(["clip255", "aniso01"]))
    w = synth.scaled(synth.WORKLOADS[LAWS[law]], n, 3, d=M * dsub, M=M, nlist=0, nprobe=0, k=k,
                     ncomp=int(r.integers(8, 60)), seed=3000 + seed, kmeans_iters=2)
    return w, k, batch, first, gamma


def draw_ivf_long(seed):
    """Inverted lists with long candidate sequences: barrier-free stretches over many lists,
    list summaries, probe selection by the library."""
    r = np.random.default_rng([777, seed])
    M = int(r.choice([16, 32, 64]))
    dsub = int(r.choice([4, 8]))
    n = int(r.integers(60_000, 200_000))
    nlist = int(r.choice([16, 40, 100, 256]))
    nprobe = int(r.integers(2, min(nlist, 70) + 1))
    k = int(r.choice([1, 10, 64, 100]))
    batch = int(r.choice([1, 16, 256, 1024]))
    gamma = float(r.choice([0.0, 0.3, 0.6]))
    law = str(r.choice(["clip255", "aniso01"]))
    w = synth.scaled(synth.WORKLOADS[LAWS[law]], n, 6, d=M * dsub, M=M, nlist=nlist, nprobe=nprobe, k=k,
                     ncomp=int(r.choice([8, 32, 128])), seed=5000 + seed, kmeans_iters=3)
    return w, k, batch, 0, gamma


def draw_mid_tables(seed):
    """Tables of 40 to 56 KB (two 768-thread workgroups per CU) with short and long rows (both
    kinds of the 80-register instance), long candidate sequences, small result sets."""
    r = np.random.default_rng([4242, seed])
    M = int(r.choice([40, 48, 56]))
    dsub = int(r.choice([2, 4, 8, 16]))
    if M * dsub % 4:
        dsub = 4
    n = int(r.integers(60_000, 160_000))
    use_ivf = bool(r.integers(0, 2))
    nlist = int(r.choice([24, 64, 150])) if use_ivf else 0
    nprobe = int(r.integers(2, min(nlist, 40) + 1)) if use_ivf else 0
    k = int(r.choice([1, 10, 33, 64]))
    batch = int(r.choice([1, 16, 100, 512, 1024, 2048]))
    gamma = float(r.choice([0.0, 0.3, 0.6]))
    law = str(r.choice(["clip255", "aniso01", "unit"]))
    w = synth.scaled(synth.WORKLOADS[LAWS[law]], n, 5, d=M * dsub, M=M, nlist=nlist, nprobe=nprobe, k=k,
                     ncomp=int(r.choice([8, 32, 128])), seed=7000 + seed, kmeans_iters=2)
    return w, k, batch, 0, gamma


@pytest.mark.parametrize("seed", list(range(48)) + [1000 + s for s in range(22)] + [2000 + s for s in range(10)] +
                         [3000 + s for s in range(10)])
def test_random_configuration(oracle, seed):
    import torch
    from paper_2508_17828_amd import trim as T
    T.lib()
    w, k, batch, _, gamma = (draw(seed) if seed < 1000 else draw_long(seed - 1000) if seed < 2000
                                 else draw_ivf_long(seed - 2000) if seed < 3000 else draw_mid_tables(seed - 3000))
    b = helpers.build(w, pq_train_max=4096, ivf_train_per_list=32)
    ix = b.index
    t = lambda a: None if a is None else torch.from_numpy(a).cuda()
    gi = T.Index(t(ix.base), t(ix.codes), t(ix.dlx), t(ix.codebooks), ids=t(ix.ids),
                 list_offsets=t(ix.list_offsets),
                 max_list_len=int(np.diff(ix.list_offsets).max()) if ix.list_offsets is not None else 0)
    if w.M % 8 == 0:
        gi.scan_head = T.trim_pack_scan_head(gi.codes, gi.dlx)
    if w.M % 16 == 0 and seed % 2 == 0:
        gi.codes_tiled = T.trim_pack_codes_tiled(gi.codes)
    if ix.list_offsets is not None and (seed % 3 != 0 or seed >= 2000):   # list-level pruning on in two draws of three
        gi.list_bounds = T.trim_pack_list_bounds(gi)
    q, probes = t(b.queries), t(b.probes)
    what = f"seed {seed}: n={w.n} d={w.d} M={w.M} k={k} batch={batch} gamma={gamma} " \
           f"nlist={w.nlist} nprobe={w.nprobe} law={w.law}"
    print(what, flush=True)
    got = T.trim_search_knn(gi, q, k, gamma, batch, probes=probes, want_mask=True)
    ref = oracle.search_knn(ix, b.queries, k, gamma, batch, b.probes, want_mask=True)
    mw = ref["mask"].shape[1]
    np.testing.assert_array_equal(got["mask"].cpu().numpy().view(np.uint32)[:, :mw], ref["mask"], err_msg=what)
    np.testing.assert_array_equal(got["n_exact"].cpu().numpy(), ref["n_exact"], err_msg=what)
    np.testing.assert_array_equal(got["ids"].cpu().numpy(), ref["ids"], err_msg=what)
    np.testing.assert_array_equal(got["d2"].cpu().numpy().view(np.uint32), ref["d2"].view(np.uint32), err_msg=what)
    radius = helpers.radius_at_percentile(b, 3.0, min(8, w.nq), 500)
    gr = T.trim_search_range(gi, q, radius, gamma, probes=probes, want_mask=True)
    rr = oracle.search_range(ix, b.queries, radius, gamma, b.probes, want_mask=True)
    np.testing.assert_array_equal(gr["offsets"].cpu().numpy(), rr["offsets"], err_msg=what)
    np.testing.assert_array_equal(gr["ids"].cpu().numpy(), rr["ids"], err_msg=what)
    np.testing.assert_array_equal(gr["d2"].cpu().numpy().view(np.uint32), rr["d2"].view(np.uint32), err_msg=what)
    np.testing.assert_array_equal(gr["mask"].cpu().numpy().view(np.uint32)[:, :mw], rr["mask"], err_msg=what)
