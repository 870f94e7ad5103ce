"""ctypes marshalling for the C ABI declared in include/rfast.h (same names)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librfast.so")
_lib = None


class RFastError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"rfast error {code}: {msg}")
        self.code = code


class RfastProblem(C.Structure):
    _fields_ = [("kind", C.c_int32), ("samples", C.c_int32), ("batch", C.c_int32), ("d", C.c_int32),
                ("K", C.c_int32), ("lam", C.c_float), ("noise_std", C.c_float), ("noise_seed", C.c_uint64),
                ("data0", C.c_void_p), ("data1", C.c_void_p)]


class RfastDiag(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("consensus_sq", "z_sq", "conservation_sq", "gsum_sq", "xbar_gap_sq",
                                           "loss_at_xbar")]


OBJECTIVES = {"diag_quadratic": 0, "least_squares": 1, "logistic": 2, "softmax_bf16": 3}
RFAST_FIELDS = {"X": 0, "Z": 1, "G": 2, "V_RING": 3, "RHO_RING": 4, "RHO_TILDE": 5, "T_NODE": 6, "TAU_R": 7,
                "TAU_C": 8, "SLOT_R": 9, "SLOT_C": 10, "ROUND": 11, "SIGMA_RING": 12, "DELIV_R": 13, "DELIV_C": 14,
                "T_HIST": 15, "SCHED_ACTIVE": 16, "SCHED_DELAY_R": 17, "SCHED_DELAY_C": 18, "SCHED_DROP_R": 19,
                "SCHED_DROP_C": 20, "SCHED_BATCH": 21, "MOMENTUM": 22}
EXPORTS = ["rfast_common_roots", "rfast_workspace_bytes", "rfast_create", "rfast_init", "rfast_round", "rfast_run", "rfast_run_generated", "rfast_run_events", "rfast_use_graphs", "rfast_use_blocks", "rfast_block_info", "rfast_set_tile_group", "rfast_sync_round", "rfast_sync_run", "rfast_rebase", "rfast_set_rebase_interval", "rfast_set_optimizer", "rfast_set_gamma_schedule", "rfast_check",
           "rfast_read_state", "rfast_write_state", "rfast_diagnostics", "rfast_diagnostics_static", "rfast_profile_enable", "rfast_kernel_time", "rfast_last_error",
           "rfast_destroy"]


def lib():
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RFastError(-6, f"{_LIB_PATH} is missing: run `python -m paper_2307_11617_amd.build`")
    L = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.rfast_workspace_bytes.restype = sz
    L.rfast_workspace_bytes.argtypes = [i32, i64, i32, i32, i32, C.POINTER(RfastProblem)]
    L.rfast_common_roots.restype = C.c_int
    L.rfast_common_roots.argtypes = [i32, vp, vp, vp, vp, vp]
    L.rfast_create.restype = C.c_int
    L.rfast_create.argtypes = [C.POINTER(vp), i32, i64, vp, vp, vp, vp, vp, vp, i32, i32, C.POINTER(RfastProblem),
                               vp, sz, vp]
    L.rfast_init.restype = C.c_int
    L.rfast_init.argtypes = [vp, vp, vp]
    L.rfast_round.restype = C.c_int
    L.rfast_round.argtypes = [vp, vp, vp, vp, vp, vp, C.c_float, vp]
    L.rfast_run.restype = C.c_int
    L.rfast_run.argtypes = [vp, i32, vp, vp, vp, vp, vp, C.c_float, vp]
    L.rfast_run_generated.restype = C.c_int
    L.rfast_run_generated.argtypes = [vp, i32, C.c_uint64, vp, i32, C.c_float, C.c_float]
    L.rfast_run_events.restype = C.c_int
    L.rfast_run_events.argtypes = [vp, i32, C.c_uint64, vp, i32, C.c_float, C.c_float]
    L.rfast_block_info.restype = C.c_int
    L.rfast_block_info.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.rfast_set_tile_group.restype = C.c_int
    L.rfast_set_tile_group.argtypes = [vp, i32]
    L.rfast_use_blocks.restype = C.c_int
    L.rfast_use_blocks.argtypes = [vp, i32]
    L.rfast_use_graphs.restype = C.c_int
    L.rfast_use_graphs.argtypes = [vp, i32]
    L.rfast_sync_round.restype = C.c_int
    L.rfast_sync_round.argtypes = [vp, C.c_float, vp]
    L.rfast_sync_run.restype = C.c_int
    L.rfast_sync_run.argtypes = [vp, i32, C.c_float, vp]
    L.rfast_rebase.restype = C.c_int
    L.rfast_rebase.argtypes = [vp]
    L.rfast_set_rebase_interval.restype = C.c_int
    L.rfast_set_rebase_interval.argtypes = [vp, i32]
    L.rfast_set_optimizer.restype = C.c_int
    L.rfast_set_optimizer.argtypes = [vp, C.c_float, C.c_float, vp]
    L.rfast_set_gamma_schedule.restype = C.c_int
    L.rfast_set_gamma_schedule.argtypes = [vp, i32, C.c_float]
    L.rfast_check.restype = C.c_int
    L.rfast_check.argtypes = [vp]
    L.rfast_read_state.restype = C.c_int
    L.rfast_read_state.argtypes = [vp, i32, vp, sz]
    L.rfast_write_state.restype = C.c_int
    L.rfast_write_state.argtypes = [vp, i32, vp, sz]
    L.rfast_diagnostics.restype = C.c_int
    L.rfast_diagnostics.argtypes = [vp, vp, C.POINTER(RfastDiag)]
    L.rfast_diagnostics_static.restype = C.c_int
    L.rfast_diagnostics_static.argtypes = [vp, vp, vp]
    L.rfast_profile_enable.restype = C.c_int
    L.rfast_profile_enable.argtypes = [vp, i32]
    L.rfast_kernel_time.restype = C.c_int
    L.rfast_kernel_time.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.rfast_last_error.restype = C.c_char_p
    L.rfast_last_error.argtypes = [vp]
    L.rfast_destroy.restype = None
    L.rfast_destroy.argtypes = [vp]
    _lib = L
    return L


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _dev_ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def rfast_last_error(ctx=None):
    return lib().rfast_last_error(ctx).decode()


def _chk(code, ctx=None):
    if code != 0:
        raise RFastError(code, rfast_last_error(ctx))


def rfast_workspace_bytes(n, p, nnzR, nnzC, D, prob):
    return int(lib().rfast_workspace_bytes(n, p, nnzR, nnzC, D, C.byref(prob)))


def rfast_common_roots(n, R_rowptr, R_col, C_rowptr, C_col):
    """Nodes that are roots of spanning trees of both G(R) and G(C^T) (Assumption 2), as a uint8 mask."""
    arrs = [np.ascontiguousarray(a, np.int32) for a in (R_rowptr, R_col, C_rowptr, C_col)]
    out = np.zeros(n, dtype=np.uint8)
    code = lib().rfast_common_roots(n, *[_np_ptr(a) for a in arrs], _np_ptr(out))
    if code < 0:
        raise RFastError(code, rfast_last_error(None))
    return out


def rfast_create(n, p, R, Cg, D, burst, prob, workspace, stream_ptr):
    """R, Cg: (rowptr int32, col int32, w float32) host numpy arrays; workspace: uint8 device tensor."""
    arrs = [np.ascontiguousarray(R[0], np.int32), np.ascontiguousarray(R[1], np.int32), np.ascontiguousarray(R[2], np.float32),
            np.ascontiguousarray(Cg[0], np.int32), np.ascontiguousarray(Cg[1], np.int32), np.ascontiguousarray(Cg[2], np.float32)]
    ctx = C.c_void_p()
    code = lib().rfast_create(C.byref(ctx), n, p, *[_np_ptr(a) for a in arrs], D, burst, C.byref(prob),
                              _dev_ptr(workspace), workspace.numel() * workspace.element_size(), C.c_void_p(stream_ptr))
    _chk(code, None)
    return ctx


def rfast_init(ctx, x0=None, batch_idx0=None):
    _chk(lib().rfast_init(ctx, _dev_ptr(x0), _dev_ptr(batch_idx0)), ctx)


def rfast_round(ctx, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx=None):
    _chk(lib().rfast_round(ctx, _dev_ptr(active), _dev_ptr(delay_R), _dev_ptr(delay_C), _dev_ptr(drop_R),
                           _dev_ptr(drop_C), gamma, _dev_ptr(batch_idx)), ctx)


def rfast_run(ctx, rounds, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx=None):
    _chk(lib().rfast_run(ctx, rounds, _dev_ptr(active), _dev_ptr(delay_R), _dev_ptr(delay_C), _dev_ptr(drop_R),
                         _dev_ptr(drop_C), gamma, _dev_ptr(batch_idx)), ctx)


def rfast_run_generated(ctx, rounds, seed, p_active, max_delay, p_drop, gamma):
    _chk(lib().rfast_run_generated(ctx, rounds, seed, _dev_ptr(p_active), max_delay, p_drop, gamma), ctx)


def rfast_run_events(ctx, iterations, seed, weights, max_delay, p_drop, gamma):
    """weights: host numpy float32 [n] or None (uniform)."""
    _chk(lib().rfast_run_events(ctx, iterations, seed, None if weights is None else _np_ptr(weights), max_delay, p_drop,
                                gamma), ctx)


def rfast_block_info(ctx, with_kind=False):
    """Lanes per node of the multi-round kernel (0: one pass per round); with_kind: also whether a
    tile belongs to one wavefront (True) or to a workgroup."""
    lanes, wave = C.c_int32(0), C.c_int32(0)
    _chk(lib().rfast_block_info(ctx, C.byref(lanes), C.byref(wave)), ctx)
    return (lanes.value, bool(wave.value)) if with_kind else lanes.value


def rfast_set_tile_group(ctx, wavefronts=0):
    _chk(lib().rfast_set_tile_group(ctx, wavefronts), ctx)


def rfast_use_blocks(ctx, on=True):
    _chk(lib().rfast_use_blocks(ctx, 2 if on == 2 else (1 if on else 0)), ctx)


def rfast_use_graphs(ctx, on=True):
    _chk(lib().rfast_use_graphs(ctx, 1 if on else 0), ctx)


def rfast_sync_round(ctx, gamma, batch_idx=None):
    _chk(lib().rfast_sync_round(ctx, gamma, _dev_ptr(batch_idx)), ctx)


def rfast_sync_run(ctx, rounds, gamma, batch_idx=None):
    _chk(lib().rfast_sync_run(ctx, rounds, gamma, _dev_ptr(batch_idx)), ctx)


def rfast_rebase(ctx):
    _chk(lib().rfast_rebase(ctx), ctx)


def rfast_set_rebase_interval(ctx, rounds):
    _chk(lib().rfast_set_rebase_interval(ctx, rounds), ctx)


def rfast_set_optimizer(ctx, momentum, weight_decay, momentum_buffer=None):
    _chk(lib().rfast_set_optimizer(ctx, momentum, weight_decay, _dev_ptr(momentum_buffer)), ctx)


def rfast_set_gamma_schedule(ctx, step_rounds, factor):
    _chk(lib().rfast_set_gamma_schedule(ctx, step_rounds, factor), ctx)


def rfast_check(ctx):
    _chk(lib().rfast_check(ctx), ctx)


def rfast_read_state(ctx, field, out):
    """out: host numpy array of exactly the field's size."""
    _chk(lib().rfast_read_state(ctx, RFAST_FIELDS[field] if isinstance(field, str) else field, _np_ptr(out), out.nbytes), ctx)
    return out


def rfast_write_state(ctx, field, src):
    """src: host numpy array of exactly the field's size and dtype."""
    src = np.ascontiguousarray(src)
    _chk(lib().rfast_write_state(ctx, RFAST_FIELDS[field] if isinstance(field, str) else field, _np_ptr(src), src.nbytes), ctx)


def rfast_diagnostics(ctx, xstar=None):
    d = RfastDiag()
    _chk(lib().rfast_diagnostics(ctx, _dev_ptr(xstar), C.byref(d)), ctx)
    return {k: getattr(d, k) for k, _ in RfastDiag._fields_}


def rfast_diagnostics_static(ctx, xstar, out):
    """out: device tensor of 6 float64; asynchronous (read it after synchronising the stream)."""
    _chk(lib().rfast_diagnostics_static(ctx, _dev_ptr(xstar), _dev_ptr(out)), ctx)


def rfast_profile_enable(ctx, on=True):
    _chk(lib().rfast_profile_enable(ctx, 1 if on else 0), ctx)


def rfast_kernel_time(ctx, which):
    ms, cnt = C.c_double(), C.c_int64()
    _chk(lib().rfast_kernel_time(ctx, which, C.byref(ms), C.byref(cnt)), ctx)
    return ms.value, cnt.value


def rfast_destroy(ctx):
    lib().rfast_destroy(ctx)


class RFast:
    """Owns the device tensors a context borrows (workspace, objective data) and
    forwards to the C ABI.  torch is used for device memory and the stream only."""

    def __init__(self, n, p, R, Cg, D, burst, objective, data0, data1, samples=0, batch=0, d=0, K=0, lam=0.0,
                 noise_std=0.0, noise_seed=0, device="cuda:0"):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.n, self.p, self.D, self.M = n, p, D, D + 2
        self.nnzR_off, self.nnzC_off = len(R[1]) - n, len(Cg[1]) - n
        self.data0 = data0.to(self.device).contiguous()
        self.data1 = data1.to(self.device).contiguous()
        kind = OBJECTIVES[objective]
        need0 = {0: n * p, 1: n * samples * p, 2: n * samples * p, 3: n * samples * d}[kind]
        need1 = n * p if kind == 0 else n * samples
        dt0 = torch.bfloat16 if kind == 3 else torch.float32
        dt1 = torch.int32 if kind == 3 else torch.float32
        if self.data0.numel() != need0 or self.data1.numel() != need1 or self.data0.dtype != dt0 or self.data1.dtype != dt1:
            raise RFastError(-1, "objective data has the wrong size or dtype")
        self.prob = RfastProblem(OBJECTIVES[objective], samples, batch, d, K, lam, noise_std, noise_seed,
                                 self.data0.data_ptr(), self.data1.data_ptr())
        nbytes = rfast_workspace_bytes(n, p, len(R[1]), len(Cg[1]), D, self.prob)
        if nbytes == 0:
            raise RFastError(-1, "sizes out of range")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self.ctx = rfast_create(n, p, R, Cg, D, burst, self.prob, self.workspace, self.stream.cuda_stream)

    def dev(self, a, dtype=None):
        t = self.torch.as_tensor(np.ascontiguousarray(a))
        if dtype is not None:
            t = t.to(dtype)
        return t.to(self.device)

    def init(self, x0=None, batch_idx0=None):
        self._keep = (None if x0 is None else self.dev(x0, self.torch.float32),
                      None if batch_idx0 is None else self.dev(batch_idx0, self.torch.int32))
        if self._keep[0] is not None and self._keep[0].numel() != self.n * self.p:
            raise RFastError(-1, "x0 must hold n*p values")
        if self._keep[1] is not None and self._keep[1].numel() != self.n * self.prob.batch:
            raise RFastError(-1, "batch_idx0 must hold n*batch rows")
        rfast_init(self.ctx, *self._keep)

    def _check_schedule(self, rounds, active, delay_R, delay_C, drop_R, drop_C, batch_idx):
        """The library cannot see the extent of device arrays: check them here, before any launch."""
        t = self.torch
        want = [("active", active, t.uint8, self.n), ("delay_R", delay_R, t.int32, self.nnzR_off),
                ("delay_C", delay_C, t.int32, self.nnzC_off), ("drop_R", drop_R, t.uint8, self.nnzR_off),
                ("drop_C", drop_C, t.uint8, self.nnzC_off)]
        if self.prob.kind != 0 and self.prob.batch > 0:
            want.append(("batch_idx", batch_idx, t.int32, self.n * self.prob.batch))
        for name, a, dt, per_round in want:
            if per_round == 0 and a is None:
                continue
            if a is None or a.dtype != dt or a.device != self.device or not a.is_contiguous() \
                    or a.numel() != rounds * per_round:
                raise RFastError(-1, f"{name}: need a contiguous {dt} tensor of {rounds * per_round} elements on {self.device}")

    def round(self, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx=None):
        self._check_schedule(1, active, delay_R, delay_C, drop_R, drop_C, batch_idx)
        rfast_round(self.ctx, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx)

    def run(self, rounds, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx=None):
        self._check_schedule(rounds, active, delay_R, delay_C, drop_R, drop_C, batch_idx)
        rfast_run(self.ctx, rounds, active, delay_R, delay_C, drop_R, drop_C, gamma, batch_idx)

    def run_generated(self, rounds, seed, p_active, max_delay, p_drop, gamma):
        t = self.torch
        if p_active.dtype != t.float32 or p_active.device != self.device or p_active.numel() != self.n \
                or not p_active.is_contiguous():
            raise RFastError(-1, "p_active: need a contiguous float32 device tensor of n probabilities")
        rfast_run_generated(self.ctx, rounds, seed, p_active, max_delay, p_drop, gamma)

    def run_events(self, iterations, seed, weights, max_delay, p_drop, gamma):
        if weights is not None:
            weights = np.ascontiguousarray(weights, dtype=np.float32)
            if weights.shape != (self.n,):
                raise RFastError(-1, "weights: need n selection weights")
        rfast_run_events(self.ctx, iterations, seed, weights, max_delay, p_drop, gamma)

    def sync_run(self, rounds, gamma, batch_idx=None):
        if self.prob.kind != 0 and self.prob.batch > 0:
            t = self.torch
            if batch_idx is None or batch_idx.dtype != t.int32 or batch_idx.device != self.device \
                    or not batch_idx.is_contiguous() or batch_idx.numel() != rounds * self.n * self.prob.batch:
                raise RFastError(-1, "batch_idx: need a contiguous int32 device tensor of rounds*n*batch rows")
        rfast_sync_run(self.ctx, rounds, gamma, batch_idx)

    def rebase(self):
        rfast_rebase(self.ctx)

    def set_optimizer(self, momentum=0.0, weight_decay=0.0):
        """Optimizer variant; init() must follow.  The buffer of the heavy-ball terms is allocated here."""
        self.momentum_buffer = None
        if momentum != 0.0:
            self.momentum_buffer = self.torch.zeros(self.n * self.p, dtype=self.torch.float32, device=self.device)
        rfast_set_optimizer(self.ctx, momentum, weight_decay, self.momentum_buffer)

    def set_gamma_schedule(self, step_rounds, factor):
        rfast_set_gamma_schedule(self.ctx, step_rounds, factor)

    def check(self):
        rfast_check(self.ctx)

    def _shape(self, field):
        n, p, M = self.n, self.p, self.M
        shapes = {"X": ((n, p), np.float32), "Z": ((n, p), np.float32), "G": ((n, p), np.float32),
                  "V_RING": ((n, M, p), np.float32), "RHO_RING": ((self.nnzC_off, M, p), np.float32),
                  "RHO_TILDE": ((self.nnzC_off, p), np.float32), "T_NODE": ((n,), np.int32),
                  "TAU_R": ((self.nnzR_off,), np.int32), "TAU_C": ((self.nnzC_off,), np.int32),
                  "SLOT_R": ((self.nnzR_off,), np.int32), "SLOT_C": ((self.nnzC_off,), np.int32),
                  "ROUND": ((1,), np.int32), "SIGMA_RING": ((n, M, p), np.float32),
                  "DELIV_R": ((self.nnzR_off,), np.uint64), "DELIV_C": ((self.nnzC_off,), np.uint64),
                  "T_HIST": ((n, self.D + 1), np.int32), "SCHED_ACTIVE": ((n,), np.uint8),
                  "SCHED_DELAY_R": ((self.nnzR_off,), np.int32), "SCHED_DELAY_C": ((self.nnzC_off,), np.int32),
                  "SCHED_DROP_R": ((self.nnzR_off,), np.uint8), "SCHED_DROP_C": ((self.nnzC_off,), np.uint8),
                  "SCHED_BATCH": ((n, self.prob.batch if self.prob.kind != 0 else 0), np.int32),
                  "MOMENTUM": ((n, p), np.float32)}
        return shapes[field]

    def read(self, field):
        shape, dt = self._shape(field)
        return rfast_read_state(self.ctx, field, np.empty(shape, dtype=dt))

    CHECKPOINT_FIELDS = ("X", "Z", "G", "V_RING", "SIGMA_RING", "RHO_TILDE", "T_NODE", "TAU_R", "TAU_C", "DELIV_R",
                         "DELIV_C", "T_HIST", "ROUND")

    def write(self, field, value):
        shape, dt = self._shape(field)
        value = np.ascontiguousarray(value, dtype=dt)
        if value.shape != shape:
            raise RFastError(-1, f"{field}: expected shape {shape}")
        rfast_write_state(self.ctx, field, value)

    def _checkpoint_fields(self):
        extra = ("MOMENTUM",) if getattr(self, "momentum_buffer", None) is not None else ()
        return self.CHECKPOINT_FIELDS + extra

    def checkpoint(self):
        return {f: self.read(f) for f in self._checkpoint_fields()}

    def restore(self, ck):
        for f in self._checkpoint_fields():
            self.write(f, ck[f])

    def diagnostics(self, xstar=None):
        return rfast_diagnostics(self.ctx, xstar)

    def close(self):
        if self.ctx is not None:
            rfast_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
