"""HIP path vs oracle for the steps in front of event-flow generation (Sec. 4.1, Sec. 4.2),
through the C ABI.  Integer work: bit-exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import gpu_harness
    return gpu_harness


def _dedup_hip(H, rec):
    import torch
    import paper_2306_08423_amd as ds
    c = H.ctx()
    n = rec.shape[0]
    d_rec = torch.from_numpy(np.ascontiguousarray(rec)).to(c.device)
    eid, rep, num, wsp = ds.alloc_dedup(c, n, c.device)
    eid.fill_(-7)
    ds.distsim_dedup_events(c, d_rec, eid, rep, num, wsp)
    torch.cuda.synchronize()
    k = int(num.cpu()[0])
    return eid.cpu().numpy()[:n], rep.cpu().numpy()[:k], k


@pytest.mark.parametrize("n,distinct,K", [(1, 1, 1), (63, 5, 2), (1025, 40, 6), (4097, 4097, 3), (300_000, 7000, 6),
                                          (70_000, 1, 16), (30_000, 500, 12), (30_000, 500, 13), (2048, 300, 5), (5000, 3, 1), (513, 513, 7), (100_000, 90_000, 4)])
def test_dedup_parity(H, n, distinct, K):
    from oracle.ingest import dedup_events
    from workloads import make_operator_records
    rec = make_operator_records(n, distinct, K=max(K, 2))[:, :K].copy()
    want_id, want_rep = dedup_events(rec)
    got_id, got_rep, k = _dedup_hip(H, rec)
    assert k == len(want_rep)
    assert (got_id == want_id).all()
    assert (got_rep == want_rep).all()


def test_dedup_all_distinct_and_empty(H):
    from oracle.ingest import dedup_events
    rec = np.arange(50_000, dtype=np.int64).reshape(-1, 1) * 7919
    got_id, got_rep, k = _dedup_hip(H, rec)
    want_id, want_rep = dedup_events(rec)
    assert k == 50_000 and (got_id == want_id).all() and (got_rep == want_rep).all()
    got_id, got_rep, k = _dedup_hip(H, np.zeros((0, 3), dtype=np.int64))
    assert k == 0


def test_dedup_is_deterministic(H):
    from workloads import make_operator_records
    rec = make_operator_records(200_000, 3000)
    a = _dedup_hip(H, rec)
    b = _dedup_hip(H, rec)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


def test_comm_event_times_parity(H):
    import torch
    import paper_2306_08423_amd as ds
    from oracle.ingest import comm_event_times
    from workloads import make_comm_profiles
    c = H.ctx()
    for n in (1, 257, 100_003):
        kind, ranks, t_a, t_b = make_comm_profiles(n)
        # the edge cases by hand: 8 / 9 devices, one device, the largest rank count, huge time
        kind[:5] = [1, 1, 1, 1, 0][: min(5, n)]
        ranks[:5] = [8, 9, 1, 2 ** 31 - 1, 2][: min(5, n)]
        t_a[:5] = [10 ** 9, 10 ** 9, 77, (1 << 61) + 3, 5][: min(5, n)]
        want = comm_event_times(kind, ranks, t_a, t_b)
        d = [torch.from_numpy(x).to(c.device) for x in (kind, ranks, t_a, t_b)]
        out = torch.full((n,), -7, dtype=torch.int64, device=c.device)
        ds.distsim_comm_event_times(c, d[0], d[1], d[2], d[3], out)
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == want).all()


def test_ingest_api_errors(H):
    import torch
    import paper_2306_08423_amd as ds
    c = H.ctx()
    rec = torch.zeros((4, 17), dtype=torch.int64, device=c.device)
    eid, rep, num, wsp = ds.alloc_dedup(c, 4, c.device)
    with pytest.raises(ds.DistSimError):
        ds.distsim_dedup_events(c, rec, eid, rep, num, wsp)                 # K above 16
    rec = torch.zeros((4, 2), dtype=torch.int64, device=c.device)
    with pytest.raises(ds.DistSimError):
        ds.distsim_dedup_events(c, rec, eid, rep, num, wsp[:16])            # workspace too small
