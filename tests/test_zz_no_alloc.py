"""es_spmm_static_ws, the entry point for callers that cannot allocate: its
output must equal es_spmm_ws's (same kernels, workspace in the library's static
device array), on two calls in a row, the second on a smaller input, and stay
inside the oracle's bound.  Collected last: the static array is shared by every
call of the process."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _graph(n, avg, seed, F):
    from workloads import random_csr
    rowptr, colidx = random_csr(n, avg, seed, empty_frac=0.05)
    rng = np.random.default_rng(seed + 1)
    vals = rng.standard_normal(colidx.size).astype(np.float32)
    X = rng.uniform(-1, 1, (n, F)).astype(np.float32)
    return rowptr, colidx, vals, X


def test_static_workspace_matches_caller_workspace_on_two_calls_in_a_row():
    import torch
    import oracle
    import paper_2104_10716_amd as es
    from gpu_util import DeviceCSR, check_Y
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    es.load_library()
    dev = "cuda:0"
    big = DeviceCSR(*_graph(60_000, 150.0, 901, 64))           # dense enough that the library partitions by itself
    small = DeviceCSR(*_graph(3_001, 40.0, 902, 41))           # smaller input right after, nothing cleared in between
    info = es.es_spmm_launch_info(big.N, big.h_colidx.size, 64, 0, "full")
    assert info["column_ranges"] == 8
    cases = [(big, 0, "full", 0, None), (small, 0, "full", 0, dict(column_partition=1)),
             (big, 300, "fastrand", 7, dict(column_partition=1)), (small, 9, "fastrand", 7, dict(column_partition=1)),
             (big, 16, "bucket", 0, None), (small, 0, "full", 0, None),
             (big, 0, "full", 0, dict(kernel=2, lanes_per_row=8)),          # flattened pieces of the column ranges
             (small, 0, "full", 0, dict(kernel=2, column_partition=1))]
    for d, W, mode, seed, opts in cases:
        what = f"static workspace N={d.N} {mode} W={W} opts={opts}"
        Ys = torch.full((d.N, d.F), float("nan"), dtype=torch.float32, device=dev)
        es.es_spmm_static_ws(d.rowptr, d.colidx, d.vals, d.X, Ys, W, mode, seed, "none", opts)
        torch.cuda.synchronize()
        ws = torch.empty(es.es_spmm_workspace_bytes(d.N) // 4, dtype=torch.int32, device=dev)
        Yw = torch.full((d.N, d.F), float("nan"), dtype=torch.float32, device=dev)
        es.es_spmm_ws(d.rowptr, d.colidx, d.vals, d.X, Yw, W, mode, seed, "none", opts, ws)
        torch.cuda.synchronize()
        assert torch.equal(Ys, Yw), what                        # same kernels, same order of sums: bit-identical
        Yref, den = oracle.spmm(d.h_rowptr, d.h_colidx, d.h_vals, d.h_X, d.F, W, mode, seed)
        check_Y(Ys.cpu().numpy(), Yref, den, what)
        del ws
    # works on another stream too (the stream orders the calls that share the array)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        Y1 = torch.empty((big.N, big.F), dtype=torch.float32, device=dev)
        Y2 = torch.empty((small.N, small.F), dtype=torch.float32, device=dev)
        es.es_spmm_static_ws(big.rowptr, big.colidx, big.vals, big.X, Y1, 0, "full")
        es.es_spmm_static_ws(small.rowptr, small.colidx, small.vals, small.X, Y2, 0, "full", 0, "none",
                             dict(column_partition=1))
    s.synchronize()
    Yref, den = oracle.spmm(big.h_rowptr, big.h_colidx, big.h_vals, big.h_X, big.F, 0, "full", 0)
    check_Y(Y1.cpu().numpy(), Yref, den, "static workspace, side stream, first call")
    Yref, den = oracle.spmm(small.h_rowptr, small.h_colidx, small.h_vals, small.h_X, small.F, 0, "full", 0)
    check_Y(Y2.cpu().numpy(), Yref, den, "static workspace, side stream, second call")


def test_static_workspace_rejects_more_rows_than_it_holds():
    import torch
    import paper_2104_10716_amd as es
    es.load_library()
    dev = "cuda:0"
    N = es.ES_SPMM_STATIC_WS_MAX_ROWS + 1
    rowptr = torch.zeros(N + 1, dtype=torch.int32, device=dev)
    colidx = torch.zeros(1, dtype=torch.int32, device=dev)
    X = torch.zeros((N, 4), dtype=torch.float32, device=dev)
    Y = torch.full((N, 4), 3.0, dtype=torch.float32, device=dev)
    with pytest.raises(es.EsSpmmError) as err:
        es.es_spmm_static_ws(rowptr, colidx, None, X, Y, 0, "full", nnz=0)
    assert err.value.status == -2 and "es_spmm_ws" in str(err.value)
    torch.cuda.synchronize()
    assert bool((Y == 3.0).all())                               # nothing was launched
    # exactly at the limit it runs (all rows empty: zeros)
    es.es_spmm_static_ws(rowptr[:N], colidx, None, X[:N - 1], Y[:N - 1], 0, "full", nnz=0)
    torch.cuda.synchronize()
    assert bool((Y[:N - 1] == 0.0).all())
