"""Helpers shared by the GPU parity tests: upload a workload, run the HIP path
through the C ABI, compare with the CPU oracle."""
import numpy as np

TOL = 1e-5      # max |Y_gpu - Y_ref| / sum_kept |a_ij| |x_j|  (the build's stated bound)


class DeviceCSR:
    def __init__(self, rowptr, colidx, vals, X, F=None, device="cuda:0"):
        import torch
        self.h_rowptr, self.h_colidx, self.h_vals, self.h_X = rowptr, colidx, vals, X
        self.rowptr = torch.from_numpy(rowptr).to(device)
        self.colidx = torch.from_numpy(colidx).to(device)
        self.vals = None if vals is None else torch.from_numpy(vals).to(device)
        self.X = torch.from_numpy(X).to(device)
        self.N = rowptr.shape[0] - 1
        self.F = X.shape[1] if F is None else F
        self.default_ws = None       # set to a workspace tensor: plain run() calls go through es_spmm_ws

    def with_workspace(self):
        """Route run() through es_spmm_ws with a workspace of this graph's size --
        the launch configuration bench.py times."""
        import torch
        import paper_2104_10716_amd as es
        self.default_ws = torch.empty(max(1, es.es_spmm_workspace_bytes(self.N) // 4), dtype=torch.int32,
                                      device=self.X.device)
        return self

    def run(self, W, mode, seed=0, ldy=None, norm=None, opts=None):
        """NaN-prefilled Y, then the product; `opts` (a dict of es_launch_opts_t
        fields) routes the call through es_spmm_ex."""
        import torch
        import paper_2104_10716_amd as es
        ldy = self.F if ldy is None else ldy
        Y = torch.full((self.N, ldy), float("nan"), dtype=torch.float32, device=self.X.device)
        if opts is None and self.default_ws is not None:
            opts = dict(workspace=self.default_ws)
        if opts is not None and "workspace" in opts:
            # es_spmm_ws: the value is a device tensor, or True = allocate one of the size the library asks for
            opts = dict(opts)
            ws = opts.pop("workspace")
            if ws is True:
                ws = torch.full((es.es_spmm_workspace_bytes(self.N) // 4,), -7, dtype=torch.int32,
                                device=self.X.device)
            es.es_spmm_ws(self.rowptr, self.colidx, self.vals, self.X, Y, W, mode, seed,
                          "none" if norm is None else norm, opts, ws, F=self.F)
        elif opts is not None:
            es.es_spmm_ex(self.rowptr, self.colidx, self.vals, self.X, Y, W, mode, seed,
                          "none" if norm is None else norm, opts, F=self.F)
        elif norm is None:
            es.es_spmm(self.rowptr, self.colidx, self.vals, self.X, Y, W, mode, seed, F=self.F)
        else:
            es.es_spmm_norm(self.rowptr, self.colidx, self.vals, self.X, Y, W, mode, seed, norm, F=self.F)
        torch.cuda.synchronize()
        return Y

    def edges(self, W, mode, seed=0, rows_per_wave=0):
        import torch
        import paper_2104_10716_amd as es
        pos, cnt = es.es_spmm_sample_edges(self.rowptr, W, mode, seed, rows_per_wave)
        torch.cuda.synchronize()
        return pos, cnt


def check_Y(Y_gpu, Yref, denom, what, tol=TOL):
    """|Y_gpu - Yref| <= tol * denom element-wise (so denom == 0 demands an exact 0)."""
    Yg = np.asarray(Y_gpu, dtype=np.float64)
    assert Yg.shape == Yref.shape, (what, Yg.shape, Yref.shape)
    assert np.isfinite(Yg).all(), f"{what}: non-finite output (unwritten rows?)"
    err = np.abs(Yg - Yref)
    bad = err > tol * denom
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol * denom), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} elements out of tolerance; "
                             f"worst at {i}: gpu={Yg[i]!r} ref={Yref[i]!r} denom={denom[i]!r}")
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(denom > 0, err / denom, 0.0)
    return float(rel.max()) if rel.size else 0.0


def check_against_oracle(d, W, mode, seed=0, rows=None, ldy=None, what="", norm=None, opts=None):
    """Run es_spmm on DeviceCSR `d` and compare (all rows, or the listed rows)."""
    import oracle
    Y = d.run(W, mode, seed, ldy=ldy, norm=norm, opts=opts)
    Yh = Y.cpu().numpy()
    if ldy is not None and ldy > d.F:
        assert np.isnan(Yh[:, d.F:]).all(), f"{what}: columns beyond F were written"
    Yh = Yh[:, :d.F]
    Yref, den = oracle.spmm(d.h_rowptr, d.h_colidx, d.h_vals, d.h_X, d.F, W, mode, seed, rows=rows,
                            norm="none" if norm is None else norm)
    if rows is not None:
        Yh = Yh[np.asarray(rows)]
    return check_Y(Yh, Yref, den, what or f"{mode} W={W} seed={seed}")


def check_every_element(d, W, mode, seed=0, what="", norm=None, opts=None, block_bytes=192 << 20):
    """Every element of Y on a graph too large for one fp64 reference: the HIP
    product once, then the oracle row block by row block (Yref + denom of a
    block stay below `block_bytes`).  Returns the largest normalised error."""
    import sys
    import time
    import oracle
    what = what or f"{mode} W={W} seed={seed}"
    Yh = d.run(W, mode, seed, norm=norm, opts=opts).cpu().numpy()
    block = max(1024, block_bytes // (16 * d.F))
    worst = 0.0
    t0 = t_last = time.perf_counter()
    for lo in range(0, d.N, block):
        hi = min(d.N, lo + block)
        rows = np.arange(lo, hi, dtype=np.int64)
        Yref, den = oracle.spmm(d.h_rowptr, d.h_colidx, d.h_vals, d.h_X, d.F, W, mode, seed, rows=rows,
                                norm="none" if norm is None else norm)
        worst = max(worst, check_Y(Yh[lo:hi, :d.F], Yref, den, f"{what} rows [{lo}, {hi})"))
        if time.perf_counter() - t_last > 30.0:                # keep a long check audibly alive
            t_last = time.perf_counter()
            print(f"  {what}: rows below {hi} of {d.N} checked ({t_last - t0:.0f} s)", flush=True)
            sys.stdout.flush()
    return worst


def check_edges(d, W, mode, seed=0, rows_per_wave=0, what=""):
    import oracle
    pos, cnt = d.edges(W, mode, seed, rows_per_wave)
    opos, ocnt = oracle.kept(d.h_rowptr, W, mode, seed)
    what = what or f"{mode} W={W} seed={seed} rpw={rows_per_wave}"
    assert np.array_equal(cnt.cpu().numpy(), ocnt), f"{what}: kept counts differ"
    assert np.array_equal(pos.cpu().numpy(), opos), f"{what}: sampled edge lists differ"


def check_backward_against_oracle(d, W, mode, seed=0, norm="none", what="", opts=None):
    """es_spmm_backward on DeviceCSR `d` (its X plays the upstream gradient dY)
    against the oracle's transposed product, every element."""
    import torch
    import oracle
    import paper_2104_10716_amd as es
    dX = torch.full((d.N, d.F), float("nan"), dtype=torch.float32, device=d.X.device)
    if opts is None:
        es.es_spmm_backward(d.rowptr, d.colidx, d.vals, d.X, dX, W, mode, seed, norm, F=d.F)
    else:
        es.es_spmm_backward_ex(d.rowptr, d.colidx, d.vals, d.X, dX, W, mode, seed, norm, opts, F=d.F)
    torch.cuda.synchronize()
    ref, den = oracle.spmm_backward(d.h_rowptr, d.h_colidx, d.h_vals, d.h_X, d.F, W, mode, seed, norm=norm)
    return check_Y(dX.cpu().numpy(), ref, den, what or f"backward {mode} W={W} seed={seed} norm={norm}")


def check_backward_pull_against_oracle(d, t, W, mode, seed=0, norm="none", what=""):
    """es_spmm_backward_pull on DeviceCSR `d` with its transposed graph `t`
    (its X plays the upstream gradient dY) against the oracle's transposed
    product, every element."""
    import torch
    import oracle
    import paper_2104_10716_amd as es
    dX = torch.full((d.N, d.F), float("nan"), dtype=torch.float32, device=d.X.device)
    es.es_spmm_backward_pull(d.rowptr, t, d.X, dX, W, mode, seed, norm, F=d.F)
    torch.cuda.synchronize()
    ref, den = oracle.spmm_backward(d.h_rowptr, d.h_colidx, d.h_vals, d.h_X, d.F, W, mode, seed, norm=norm)
    return check_Y(dX.cpu().numpy(), ref, den, what or f"backward pull {mode} W={W} seed={seed} norm={norm}")
