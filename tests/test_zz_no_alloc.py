"""avq_search_noalloc (the entry point for callers that cannot allocate device memory) against
avq_search, through the C ABI: same ids and scores, bit for bit, on calls in a row that share
the library's static scratch array -- the second with a smaller input, then another index."""
import ctypes as C

import numpy as np
import pytest

import synth_inputs as si
from util import unit_rows

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
avq = pytest.importorskip("paper_1908_10396_amd")


def _index(n, d, M, bits, seed):
    rng = np.random.default_rng(seed)
    x = unit_rows(rng, n, d)
    xd = torch.from_numpy(x).cuda()
    idx = avq.Index(d, M, bits, T=0.2, kmeans_iters=4, encode_passes=3, seed=seed)
    idx.train(xd[: min(n, 20000)])
    idx.encode(xd)
    return idx, xd


def _raw_noalloc(idx, qd, k, R, lut_mode):
    """The call as a C program would make it: raw pointers, caller-owned outputs."""
    nq = qd.shape[0]
    ids = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
    sc = torch.full((nq, k), float("nan"), dtype=torch.float32, device="cuda")
    rc = avq.lib().avq_search_noalloc(idx._h, C.c_void_p(qd.data_ptr()), nq, k, R, lut_mode,
                                      C.c_void_p(ids.data_ptr()), C.c_void_p(sc.data_ptr()),
                                      C.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc, ids, sc


@pytest.mark.parametrize("bits,M,d", [(4, 50, 100), (8, 8, 64)])
def test_noalloc_equals_search_on_consecutive_calls(bits, M, d):
    idx_a, xa = _index(70_001, d, M, bits, seed=11)
    idx_b, xb = _index(9_000, d, M, bits, seed=12)          # the smaller input
    rng = np.random.default_rng(5)
    q = torch.from_numpy(unit_rows(rng, 32, d)).cuda()
    # the first call on a device looks the scratch array's address up (the runtime maps the library's
    # device globals at that point); from then on free device memory must not move
    rc, _, _ = _raw_noalloc(idx_b, q[:1].contiguous(), 1, 0, avq.LUT_F32)
    assert rc == avq.AVQ_OK, avq.lib().avq_last_error()
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    calls = [(idx_a, q[:7], 10, 100), (idx_b, q[:3], 10, 40), (idx_a, q[:1], 5, 0), (idx_b, q[:32], 10, 100),
             (idx_a, q[5:6], 10, 100)]
    got = []
    for lut_mode in (avq.LUT_F32, avq.LUT_U8):
        for idx, qd, k, R in calls:
            rc, ids, sc = _raw_noalloc(idx, qd.contiguous(), k, R, lut_mode)
            assert rc == avq.AVQ_OK, avq.lib().avq_last_error()
            got.append((ids, sc))
    torch.cuda.synchronize()
    # nothing was allocated on the device by those calls (the outputs above come from torch's cache or
    # from fresh blocks torch itself asked for: compare what the library could have taken)
    assert torch.cuda.mem_get_info()[0] >= free0 - (8 << 20)
    it = iter(got)
    for lut_mode in (avq.LUT_F32, avq.LUT_U8):
        for idx, qd, k, R in calls:
            ids, sc = next(it)
            wi, ws = idx.search(qd.contiguous(), k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), wi.cpu().numpy())
            np.testing.assert_array_equal(sc.cpu().numpy(), ws.cpu().numpy())
            assert ids.min().item() >= 0
    # the same with the selection of the blocks and the exact re-scoring spread over several workgroups per
    # query (launch shapes of large indexes: their counters live in the scratch array too)
    for idx in (idx_a, idx_b):
        idx.set_tuning("select_split", 16)
        idx.set_tuning("rerank_split", 12)
    for lut_mode in (avq.LUT_F32, avq.LUT_U8):
        for idx, qd, k, R in calls:
            rc, ids, sc = _raw_noalloc(idx, qd.contiguous(), k, R, lut_mode)
            assert rc == avq.AVQ_OK, avq.lib().avq_last_error()
            for name in ("select_split", "rerank_split"):
                idx.set_tuning(name, 1)
            wi, ws = idx.search(qd.contiguous(), k, R, lut_mode)
            idx.set_tuning("select_split", 16)
            idx.set_tuning("rerank_split", 12)
            np.testing.assert_array_equal(ids.cpu().numpy(), wi.cpu().numpy())
            np.testing.assert_array_equal(sc.cpu().numpy(), ws.cpu().numpy())
    idx_a.close()
    idx_b.close()


def test_noalloc_rejects_what_it_cannot_serve():
    idx, xd = _index(5_000, 32, 16, 4, seed=3)
    q = torch.from_numpy(unit_rows(np.random.default_rng(1), 40, 32)).cuda()
    rc, _, _ = _raw_noalloc(idx, q, 10, 100, avq.LUT_F32)                 # 40 queries: above the limit
    assert rc == avq.AVQ_EINVAL and b"at most" in avq.lib().avq_last_error()
    rc, _, _ = _raw_noalloc(idx, q[:4].contiguous(), 10, 5, avq.LUT_F32)  # reorder_k < k
    assert rc == avq.AVQ_EINVAL
    idx.close()
    # a partitioned index
    cfg = si.CONFIGS["tiny"]
    x = si.make_data(cfg, 4000)
    xd = torch.from_numpy(x).cuda()
    ivf = avq.Index(cfg["d"], cfg["M"], cfg["bits"], T=0.2, n_leaves=8, kmeans_iters=3, leaf_kmeans_iters=3,
                    encode_passes=2)
    ivf.train(xd)
    ivf.encode(xd)
    rc, _, _ = _raw_noalloc(ivf, q[:2].contiguous(), 10, 100, avq.LUT_F32)
    assert rc == avq.AVQ_EINVAL and b"flat" in avq.lib().avq_last_error()
    ivf.close()


def test_noalloc_scratch_limit_is_enforced_on_the_host():
    # 32 queries x 2,000,000 stored points need 8 * 32 * 7,813 blocks = 2 MB of block maxima: fine; the
    # candidate keys of reorder_k = 512 need 32 * 256 * 512 * 8 = 33.5 MB: fine; both with 8-bit codes of
    # 64 subspaces (tables 2 MB) still fit. A synthetic code array large enough to exceed 64 MiB:
    # 32 queries x 300,000 blocks x 8 B = 76.8 MB.
    n = 300_000 * 256
    codes = torch.zeros((n, 1), dtype=torch.uint8, device="cuda")
    idx = avq.Index(2, 1, 8, T=0.2)
    idx.set_codebooks(np.zeros((1, 256, 2), np.float32))
    idx.set_database(None, codes)
    q = torch.zeros((32, 2), dtype=torch.float32, device="cuda")
    rc, _, _ = _raw_noalloc(idx, q, 10, 0, avq.LUT_F32)
    assert rc == avq.AVQ_EINVAL and b"scratch" in avq.lib().avq_last_error()
    rc, ids, _ = _raw_noalloc(idx, q[:8].contiguous(), 10, 0, avq.LUT_F32)   # 19.2 MB: served
    assert rc == avq.AVQ_OK
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ids.cpu().numpy(), np.tile(np.arange(10, dtype=np.int32), (8, 1)))
    idx.close()


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_noalloc_under_graph_capture_replays_like_eager_calls(lut_mode):
    # one of the callers the entry point is for: its launches recorded into a HIP graph (no allocation, no
    # memset nodes), replayed with other work of the program between the replays, every replay against avq_search
    if not hasattr(torch.cuda, "CUDAGraph"):
        pytest.skip("this torch has no graph capture")
    idx, _ = _index(70_001, 100, 50, 4, seed=21)
    rng = np.random.default_rng(6)
    q = torch.from_numpy(unit_rows(rng, 6, 100)).cuda()
    k, R = 10, 100
    ids = torch.empty((1, k), dtype=torch.int32, device="cuda")
    sc = torch.empty((1, k), dtype=torch.float32, device="cuda")
    qbuf = q[0:1].clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(3):   # first calls: symbol look-up, kernel attributes -- none of that inside the capture
            idx.search_noalloc(qbuf, k, R, lut_mode, out=(ids, sc))
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        idx.search_noalloc(qbuf, k, R, lut_mode, out=(ids, sc))
    for i in range(6):
        qbuf.copy_(q[i:i + 1])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_ids, got_sc = ids.clone(), sc.clone()
        want_ids, want_sc = idx.search(q[i:i + 1].contiguous(), k, R, lut_mode)   # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(got_ids, want_ids), i
        assert torch.equal(got_sc, want_sc), i
    idx.close()
