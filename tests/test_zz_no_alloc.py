"""trim_search_range_static (the range search that allocates nothing: the workspace is the
library's own scratch area) against trim_search_range, through the C ABI: two calls in a row,
the second on a smaller input, so that whatever the first call left in the scratch area would
show; every output of either call must equal the workspace variant's bit for bit, and the
workspace variant is compared with the oracle."""
import ctypes as C

import numpy as np
import pytest

from tests import helpers

pytestmark = pytest.mark.gpu


def _gpu_index(b):
    import torch
    from paper_2508_17828_amd import trim
    g = lambda a: None if a is None else torch.from_numpy(a).cuda()
    ix = b.index
    lens = np.diff(ix.list_offsets) if ix.list_offsets is not None else np.array([0])
    return trim.Index(g(ix.base), g(ix.codes), g(ix.dlx), g(ix.codebooks), ids=g(ix.ids),
                      list_offsets=g(ix.list_offsets), max_list_len=int(lens.max()))


def _same(a, b):
    for key in ("offsets", "ids", "d2", "n_scanned", "n_exact", "mask"):
        x, y = a[key].cpu().numpy(), b[key].cpu().numpy()
        np.testing.assert_array_equal(x.view(np.uint32) if x.dtype == np.float32 else x,
                                      y.view(np.uint32) if y.dtype == np.float32 else y, err_msg=key)
    assert a["required"] == b["required"]


def test_static_scratch_equals_workspace_variant_twice(oracle):
    import torch
    from paper_2508_17828_amd import trim
    L = trim.lib()
    assert L.trim_static_scratch_bytes() == 32 * 1024 * 1024
    b = helpers.cached("C2", 60_000, 96, 64, 8)
    gix = _gpu_index(b)
    gq, gp = torch.from_numpy(b.queries).cuda(), torch.from_numpy(b.probes).cuda()
    radius = helpers.radius_at_percentile(b, 0.5)
    # first call: all 96 queries; second call: fewer queries, fewer probed lists, smaller radius
    first = dict(q=gq, p=gp, radius=radius, gamma=0.3)
    second = dict(q=gq[5:45].contiguous(), p=gp[5:45, :3].contiguous(), radius=0.8 * radius, gamma=0.0)
    outs = []
    for c in (first, second):
        outs.append(trim.trim_search_range(gix, c["q"], c["radius"], c["gamma"], probes=c["p"],
                                           want_mask=True, static_scratch=True))
    torch.cuda.synchronize()
    for c, got in zip((first, second), outs):
        ref = trim.trim_search_range(gix, c["q"], c["radius"], c["gamma"], probes=c["p"], want_mask=True)
        _same(got, ref)
        assert got["required"] > 0
        orc = oracle.search_range(b.index, np.ascontiguousarray(c["q"].cpu().numpy()), c["radius"],
                                  c["gamma"], np.ascontiguousarray(c["p"].cpu().numpy()))
        np.testing.assert_array_equal(got["offsets"].cpu().numpy(), orc["offsets"])
        np.testing.assert_array_equal(got["ids"].cpu().numpy(), orc["ids"])


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    from paper_2508_17828_amd import trim
    L = trim.lib()
    b = helpers.cached("C2", 60_000, 96, 64, 8)
    gix = _gpu_index(b)
    # all n scanned by 4096 queries: 4096 x 60,000 pairs need far more than 32 MiB
    nq = 4096
    assert L.trim_range_workspace_bytes(nq, gix.n) > L.trim_static_scratch_bytes()
    q = torch.zeros((nq, gix.d), dtype=torch.float32, device="cuda")
    with pytest.raises(trim.TrimError) as e:
        trim.trim_search_range(gix, q, 1.0, 0.0, static_scratch=True)
    assert e.value.status == -3 and "TRIM_STATIC_SCRATCH_BYTES" in str(e.value)
    # the workspace variant still works right after the refusal
    r = trim.trim_search_range(gix, q[:4].contiguous(), 1.0, 0.0)
    assert r["required"] >= 0
