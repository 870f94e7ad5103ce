"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the header declares, sizes its workspace, and rejects malformed
graphs and parameters before any device work (Assumptions 1 and 2)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2307_11617_amd as rf
from paper_2307_11617_amd.binding import RfastProblem
from rfast_workloads import graphs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_DEV = 1 << 20  # never dereferenced: every case below fails validation first


def _declared():
    text = open(os.path.join(ROOT, "include", "rfast.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rfast_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared()
    assert {"rfast_create", "rfast_round", "rfast_read_state", "rfast_init", "rfast_run"} <= set(names)
    L = rf.lib()
    for name in names:
        assert hasattr(L, name), name


def _prob(kind=0, **kw):
    p = RfastProblem(kind, kw.get("samples", 0), kw.get("batch", 0), kw.get("d", 0), kw.get("K", 0), 0.0, 0.0, 0,
                     FAKE_DEV, FAKE_DEV)
    return p


def test_workspace_bytes_is_pure_and_checks_ranges():
    pr = _prob()
    a = rf.rfast_workspace_bytes(16, 1 << 20, 48, 48, 7, pr)
    b = rf.rfast_workspace_bytes(16, 1 << 21, 48, 48, 7, pr)
    # x, z, 2 g, 9-slot v ring and 9-slot running-sum ring per node, 32 rho~ vectors, the node average
    vectors = 16 * (1 + 1 + 2 + 9 + 9) + 32 + 1
    assert a >= vectors * (1 << 20) * 4 and a - vectors * (1 << 20) * 4 < 1 << 20
    assert b - a == vectors * (1 << 20) * 4
    assert rf.rfast_workspace_bytes(16, 0, 48, 48, 7, pr) == 0
    assert rf.rfast_workspace_bytes(16, 64, 48, 48, 63, pr) == 0           # D + 2 > 64
    assert rf.rfast_workspace_bytes(16, 64, 8, 48, 7, pr) == 0             # fewer entries than self-loops
    assert rf.rfast_workspace_bytes(4, 64 * 32, 8, 8, 3, _prob(3, samples=128, batch=64, d=64, K=32)) > 0
    assert rf.rfast_workspace_bytes(4, 60 * 32, 8, 8, 3, _prob(3, samples=128, batch=64, d=60, K=32)) == 0


def _create(wr, wc, D=5, burst=2, p=64, prob=None, ws_ptr=FAKE_DEV, ws_bytes=1 << 40, raw=None):
    R, Cg = graphs.from_dense(wr), graphs.from_dense(wc)
    arrs = [R.rowptr, R.col, R.w32(), Cg.rowptr, Cg.col, Cg.w32()]
    if raw:
        arrs = raw(arrs)
    arrs = [np.ascontiguousarray(a) for a in arrs]
    ctx = C.c_void_p()
    prob = prob or _prob()
    code = rf.lib().rfast_create(C.byref(ctx), R.n, p, *[a.ctypes.data_as(C.c_void_p) for a in arrs], D, burst,
                                 C.byref(prob), C.c_void_p(ws_ptr), ws_bytes, None)
    assert not ctx.value
    return code, rf.rfast_last_error(None)


def test_create_rejects_non_stochastic_weights():
    wr, wc = graphs.directed_ring(5)
    bad = wr.copy()
    bad[2, 2] = 0.6
    code, msg = _create(bad, wc)
    assert code == -2 and "row 2" in msg
    bad = wc.copy()
    bad[3, 2] = 0.4          # column 2 now sums to 0.9
    code, msg = _create(wr, bad)
    assert code == -2 and "column 2" in msg
    bad = wr.copy()
    bad[1, 1] = 0.0
    bad[1, 0] = 1.0          # row still sums to one but the self-loop is gone
    code, msg = _create(bad, wc)
    assert code == -2 and "self-loop" in msg


def test_create_rejects_negative_weight_and_malformed_csr():
    wr, wc = graphs.bidirectional_ring(5)

    def neg(arrs):
        w = arrs[2].copy()
        w[0], w[1] = -0.2, w[1] + w[0] + 0.2
        arrs[2] = w
        return arrs
    code, msg = _create(wr, wc, raw=neg)
    assert code == -2 and "positive" in msg

    def unsorted(arrs):
        col = arrs[1].copy()
        col[0], col[1] = col[1], col[0]
        arrs[1] = col
        return arrs
    code, msg = _create(wr, wc, raw=unsorted)
    assert code == -3 and "ascending" in msg


def test_create_rejects_graphs_without_common_root():
    n = 5
    r, c = graphs.line_tree(n)           # R pulls away from root 0, C pushes towards 0: common root 0
    code, _ = _create(r, c, ws_bytes=0)
    assert code == -5                    # passes the graph checks, then the workspace is too small
    c_wrong = np.zeros((n, n))           # C pushes away from 0: the only sink is n-1
    c_wrong[n - 1, n - 1] = 1.0
    for j in range(n - 1):
        c_wrong[j, j] = 0.5
        c_wrong[j + 1, j] = 0.5
    code, msg = _create(r, c_wrong)
    assert code == -3 and "Assumption 2" in msg


def test_create_rejects_bad_parameters():
    wr, wc = graphs.directed_ring(4)
    assert _create(wr, wc, D=63)[0] == -4
    assert _create(wr, wc, D=3, burst=5)[0] == -4
    assert _create(wr, wc, D=3, burst=0)[0] == -4
    assert _create(wr, wc, ws_ptr=FAKE_DEV + 8)[0] == -1       # misaligned workspace
    assert _create(wr, wc, ws_bytes=1024)[0] == -5
    assert _create(wr, wc, p=64, prob=_prob(1, samples=0))[0] == -1
    assert _create(wr, wc, p=64 * 32, prob=_prob(3, samples=128, batch=96, d=64, K=32))[0] == -1


def test_null_context_calls_fail_cleanly():
    L = rf.lib()
    assert L.rfast_init(None, None, None) == -1
    assert L.rfast_round(None, None, None, None, None, None, 0.1, None) == -1
    assert L.rfast_check(None) == -1
    assert L.rfast_set_optimizer(None, 0.9, 0.0, None) == -1
    assert L.rfast_set_gamma_schedule(None, 10, 0.5) == -1
    assert L.rfast_run_generated(None, 1, 0, None, 0, 0.0, 0.1) == -1
    assert L.rfast_run_events(None, 1, 0, None, 0, 0.0, 0.1) == -1
    assert L.rfast_set_rebase_interval(None, 10) == -1
    assert L.rfast_use_blocks(None, 1) == -1
    assert L.rfast_block_info(None, None, None) == -1
    assert L.rfast_write_state(None, 0, None, 0) == -1
    L.rfast_destroy(None)


def test_common_roots_of_named_topologies():
    def roots(build, n):
        r, c = build(n)
        R, Cg = graphs.from_dense(r), graphs.from_dense(c)
        return rf.rfast_common_roots(n, R.rowptr, R.col, Cg.rowptr, Cg.col).nonzero()[0].tolist()
    assert roots(graphs.tree_pull_star_push, 9) == [0]
    assert roots(graphs.line_tree, 6) == [0]
    assert roots(graphs.directed_ring, 5) == [0, 1, 2, 3, 4]
    assert roots(graphs.exponential, 8) == list(range(8))
    assert roots(graphs.binary_tree, 7) == [0]
    assert roots(graphs.binary_tree, 10) == [0]
    assert roots(graphs.mesh, 7) == list(range(7))          # 3 columns, short last row
    assert roots(lambda n: graphs.multi_root_split(n, 3), 11) == [0, 1, 2]
    assert roots(lambda n: graphs.multi_root_split(n, 1), 5) == [0]
    # two roots: nodes 0 and 1 exchange both ways, node 2 only listens / only sends
    r = np.array([[.5, .5, 0], [.5, .5, 0], [0, .5, .5]])
    c = np.array([[.5, .25, .25], [.5, .5, .25], [0, .25, .5]])
    R, Cg = graphs.from_dense(r), graphs.from_dense(c)
    assert rf.rfast_common_roots(3, R.rowptr, R.col, Cg.rowptr, Cg.col).tolist() == [1, 1, 0]
    # R rooted at 0 but C pushing away from 0: no common root
    n = 4
    rr, _ = graphs.line_tree(n)
    cw = np.zeros((n, n))
    cw[n - 1, n - 1] = 1.0
    for j in range(n - 1):
        cw[j, j] = cw[j + 1, j] = 0.5
    R, Cg = graphs.from_dense(rr), graphs.from_dense(cw)
    assert rf.rfast_common_roots(n, R.rowptr, R.col, Cg.rowptr, Cg.col).sum() == 0
