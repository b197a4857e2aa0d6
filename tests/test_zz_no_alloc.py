"""The entry point that allocates nothing (distsim_search_static) against distsim_search, through the
C ABI: two calls in a row, the second on a smaller input, both objectives; every output word equal."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

INT64_MAX = np.iinfo(np.int64).max


def _inputs(rng, n):
    b = rng.integers(1, 1 << 52, n)
    b[rng.integers(0, n, n // 3 + 1)] = b[n // 2]            # ties
    b[rng.random(n) < 0.1] = INT64_MAX                       # invalid candidates
    return b, rng.integers(-2, 1 << 20, n)


def test_search_static_equals_search_on_two_calls_in_a_row(oracle_mod):
    import ctypes as C
    import torch
    import paper_2306_08423_amd as ds
    print("[case] distsim_search_static, 3000001 then 1000 candidates, both objectives", flush=True)
    ctx = ds.Context(0)
    lib, dev = ctx.lib, ctx.device
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(77)
    for obj in (0, 1):
        for n in (3_000_001, 1000):                          # the second call reads fewer partial results than the first wrote
            b, wg = _inputs(rng, n)
            d_b, d_w = torch.from_numpy(b).to(dev), torch.from_numpy(wg).to(dev)
            want = torch.full((2,), -7, dtype=torch.int64, device=dev)
            got = torch.full((2,), -7, dtype=torch.int64, device=dev)
            scratch = torch.empty(lib.distsim_search_scratch_bytes(n), dtype=torch.uint8, device=dev)
            rc = lib.distsim_search(ctx.h, C.c_void_p(d_b.data_ptr()), C.c_void_p(d_w.data_ptr()), n, obj,
                                    C.c_void_p(want.data_ptr()), C.c_void_p(scratch.data_ptr()), stream)
            assert rc == 0, lib.distsim_last_error(ctx.h)
            rc = lib.distsim_search_static(ctx.h, C.c_void_p(d_b.data_ptr()), C.c_void_p(d_w.data_ptr()), n, obj,
                                           C.c_void_p(got.data_ptr()), stream)
            assert rc == 0, lib.distsim_last_error(ctx.h)
            torch.cuda.synchronize()
            assert got.cpu().tolist() == want.cpu().tolist(), (obj, n)
            assert tuple(got.cpu().tolist()) == oracle_mod.search(b, wg, obj), (obj, n)
    # nothing left to choose from, and an empty list
    none = torch.full((100,), INT64_MAX, dtype=torch.int64, device=dev)
    got = torch.full((2,), -7, dtype=torch.int64, device=dev)
    assert lib.distsim_search_static(ctx.h, C.c_void_p(none.data_ptr()), None, 100, 0, C.c_void_p(got.data_ptr()), stream) == 0
    torch.cuda.synchronize()
    assert got.cpu().tolist() == [-1, INT64_MAX]
    assert lib.distsim_search_static(ctx.h, None, None, 0, 0, C.c_void_p(got.data_ptr()), stream) == 0
    torch.cuda.synchronize()
    assert got.cpu().tolist() == [-1, INT64_MAX]
    # sizes beyond the stated maximum and bad arguments are errors, not launches
    assert lib.distsim_search_static(ctx.h, C.c_void_p(none.data_ptr()), None, 1 << 31, 0, C.c_void_p(got.data_ptr()), stream) == -4
    assert b"DISTSIM_SEARCH_STATIC_MAX_C" in lib.distsim_last_error(ctx.h)
    assert lib.distsim_search_static(ctx.h, C.c_void_p(none.data_ptr()), None, 100, 1, C.c_void_p(got.data_ptr()), stream) == -1
    assert lib.distsim_search_static(ctx.h, C.c_void_p(none.data_ptr()), None, 100, 0, None, stream) == -1
    # a second context on the same GPU finds the same array
    ctx2 = ds.Context(0)
    b, wg = _inputs(rng, 70_000)
    d_b = torch.from_numpy(b).to(dev)
    assert lib.distsim_search_static(ctx2.h, C.c_void_p(d_b.data_ptr()), None, 70_000, 0, C.c_void_p(got.data_ptr()), stream) == 0
    torch.cuda.synchronize()
    assert tuple(got.cpu().tolist()) == oracle_mod.search(b, None, 0)
    ctx2.close()
    ctx.close()
