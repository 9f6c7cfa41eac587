"""ctypes binding of libqsr.so: same names as the C ABI in include/qsr.h, argument marshalling
only.  PyTorch supplies device memory and the stream; no step of the method runs in Python."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = os.path.join(_HERE, "libqsr.so")
_lib = None

EXPORTS = ["qsr_validate", "qsr_workspace_bytes", "qsr_host_schedule", "qsr_init", "qsr_local_step", "qsr_maybe_sync",
           "qsr_run", "qsr_get_H", "qsr_get_state", "qsr_set_state", "qsr_read_sync_log", "qsr_read_host_schedule", "qsr_eta_table", "qsr_read_loss", "qsr_restart",
           "qsr_timing", "qsr_read_timing", "qsr_read_timing_stats", "qsr_destroy", "qsr_average_rows", "qsr_clip_workspace_bytes", "qsr_clip_factors", "qsr_clip_factors_static", "qsr_strerror",
           "qsr_last_hip_error"]

OPTS = {"sgdm": 0, "adamw": 1}
LRS = {"cosine": 0, "step": 1, "table": 2, "linear": 3, "pow2cos": 4}
MODELS = {"external": 0, "noise": 1, "linreg": 2, "mlp2": 3, "resmlp": 4}


class QSRError(RuntimeError):
    def __init__(self, code, what=""):
        self.code = code
        msg = lib().qsr_strerror(code).decode()
        if code == -3:
            msg += " (hipError %d)" % lib().qsr_last_hip_error()
        super().__init__("%s: %s [%d]" % (what, msg, code))


class Config(C.Structure):
    _fields_ = [
        ("K", C.c_int32), ("opt", C.c_int32), ("model", C.c_int32), ("lr_kind", C.c_int32),
        ("H_base", C.c_int32), ("n_milestones", C.c_int32), ("n_blocks", C.c_int32),
        ("power", C.c_int32), ("parallel", C.c_int32), ("average_state", C.c_int32),
        ("fuse_sync", C.c_int32), ("n_heads", C.c_int32), ("fuse_gradient", C.c_int32), ("reserved", C.c_int32),
        ("P", C.c_int64), ("T", C.c_int64), ("T_warm", C.c_int64), ("t_local_start", C.c_int64),
        ("t_swap_start", C.c_int64), ("B_loc", C.c_int64),
        ("d_in", C.c_int64), ("d_hidden", C.c_int64), ("d_out", C.c_int64), ("seq_len", C.c_int64),
        ("momentum", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
        ("weight_decay", C.c_double), ("eta_max", C.c_double), ("eta_min", C.c_double),
        ("step_factor", C.c_double), ("alpha", C.c_double), ("grad_sigma", C.c_double),
        ("data_sigma", C.c_double), ("clip_norm", C.c_double),
        ("seed", C.c_uint64),
        ("milestones", C.c_void_p), ("eta_table", C.c_void_p), ("stream", C.c_void_p),
    ]


def lib_path():
    return _LIB


def lib():
    """Loads the built library; fails loudly if it is not there (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RuntimeError("libqsr.so is not built: run `python -m paper_2310_14423_amd.build`")
        L = C.CDLL(_LIB)
        L.qsr_strerror.restype = C.c_char_p
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise QSRError(rc, what)


def make_config(w, stream=0, eta_table=None):
    """qsr_config from a workload dictionary (see workloads.py).  Returns (config, keepalive)."""
    keep = []
    c = Config()
    c.K = w["K"]; c.opt = OPTS[w["opt"]]; c.model = MODELS[w["model"]]
    c.H_base = w["H_base"]; c.alpha = w["alpha"]
    c.power = w.get("power", 2); c.parallel = int(w.get("parallel", False))
    c.t_local_start = w.get("t_local_start", 0)
    c.t_swap_start = w.get("t_swap_start", 0)
    c.average_state = int(w.get("average_state", False))
    c.fuse_sync = int(w.get("fuse_sync", False))
    c.clip_norm = float(w.get("clip_norm", 0.0))
    c.P = w["P"]; c.T = w["T"]; c.T_warm = w.get("T_warm", 0)
    c.B_loc = w.get("B_loc", 0); c.d_in = w.get("d_in", 0); c.d_hidden = w.get("d_hidden", 0)
    c.d_out = w.get("d_out", 0); c.n_blocks = w.get("n_blocks", 0)
    c.n_heads = w.get("n_heads", 0); c.seq_len = w.get("seq_len", 0)
    c.fuse_gradient = int(w.get("fuse_gradient", 0))
    c.momentum = w.get("mu", 0.0); c.beta1 = w.get("beta1", 0.9); c.beta2 = w.get("beta2", 0.999)
    c.eps = w.get("eps", 1e-8); c.weight_decay = w.get("lam", 0.0)
    c.grad_sigma = w.get("grad_sigma", 0.0); c.data_sigma = w.get("data_sigma", 0.0)
    c.seed = w.get("seed", 0)
    c.stream = stream
    if eta_table is not None:
        tab = np.ascontiguousarray(eta_table, dtype=np.float64)
        keep.append(tab)
        c.lr_kind = LRS["table"]; c.eta_table = tab.ctypes.data
    else:
        c.lr_kind = LRS[w["lr"]]
        c.eta_max = w["eta_max"]; c.eta_min = w.get("eta_min", 0.0)
        if w["lr"] == "step":
            ms = np.ascontiguousarray(w["milestones"], dtype=np.int64)
            keep.append(ms)
            c.milestones = ms.ctypes.data; c.n_milestones = len(ms); c.step_factor = w["factor"]
    return c, keep


def validate(cfg):
    why = C.c_char_p()
    rc = lib().qsr_validate(C.byref(cfg), C.byref(why))
    return rc, (why.value or b"").decode()


def workspace_bytes(cfg):
    n = C.c_size_t(0)
    _check(lib().qsr_workspace_bytes(C.byref(cfg), C.byref(n)), "qsr_workspace_bytes")
    return n.value


def host_schedule(cfg):
    """(averaging points, periods) of a whole run, from the library's host-side schedule routine."""
    n = C.c_int64()
    _check(lib().qsr_host_schedule(C.byref(cfg), None, None, C.c_int64(0), C.byref(n)), "qsr_host_schedule")
    t = np.zeros(max(n.value, 1), dtype=np.int64); H = np.zeros_like(t)
    _check(lib().qsr_host_schedule(C.byref(cfg), t.ctypes.data_as(C.c_void_p), H.ctypes.data_as(C.c_void_p),
                                   C.c_int64(n.value), C.byref(n)), "qsr_host_schedule")
    return t[:n.value], H[:n.value]


def average_rows(buf, stream=None):
    """buf: 2-D float32 CUDA tensor [K][P], averaged over K in place (all rows get the mean)."""
    import torch
    assert buf.is_cuda and buf.dtype == torch.float32 and buf.is_contiguous() and buf.dim() == 2
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _check(lib().qsr_average_rows(C.c_void_p(buf.data_ptr()), C.c_int32(buf.shape[0]),
                                  C.c_int64(buf.shape[1]), C.c_void_p(st)), "qsr_average_rows")


def clip_factors(grads, max_norm, stream=None):
    """grads: 2-D float32 CUDA tensor [K][P].  Returns (coef, norm), float32 CUDA tensors of K entries:
    the per-worker clipping factors min(1, max_norm / (||g_k|| + 1e-6)) and the norms."""
    import torch
    assert grads.is_cuda and grads.dtype == torch.float32 and grads.is_contiguous() and grads.dim() == 2
    K, P = grads.shape
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    n = C.c_size_t(0)
    _check(lib().qsr_clip_workspace_bytes(C.c_int32(K), C.c_int64(P), C.byref(n)), "qsr_clip_workspace_bytes")
    ws = torch.empty(max(n.value // 8, 1), dtype=torch.float64, device=grads.device)
    coef = torch.empty(K, dtype=torch.float32, device=grads.device)
    norm = torch.empty(K, dtype=torch.float32, device=grads.device)
    _check(lib().qsr_clip_factors(C.c_void_p(grads.data_ptr()), C.c_int32(K), C.c_int64(P), C.c_float(max_norm),
                                  C.c_void_p(ws.data_ptr()), C.c_size_t(n.value), C.c_void_p(coef.data_ptr()),
                                  C.c_void_p(norm.data_ptr()), C.c_void_p(st)), "qsr_clip_factors")
    return coef, norm


def clip_factors_static(grads, max_norm, coef, norm, stream=None):
    """qsr_clip_factors_static: results into the caller's coef and norm tensors (K floats each); the
    library allocates nothing."""
    import torch
    assert grads.is_cuda and grads.dtype == torch.float32 and grads.is_contiguous() and grads.dim() == 2
    K, P = grads.shape
    assert coef.is_cuda and norm.is_cuda and coef.dtype == norm.dtype == torch.float32 and coef.numel() >= K <= norm.numel()
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _check(lib().qsr_clip_factors_static(C.c_void_p(grads.data_ptr()), C.c_int32(K), C.c_int64(P), C.c_float(max_norm),
                                         C.c_void_p(coef.data_ptr()), C.c_void_p(norm.data_ptr()), C.c_void_p(st)),
           "qsr_clip_factors_static")


def _allocate_state(torch, dev, K, P, second_moment, placement):
    """The [K][P] arrays params, grads, state0, state1 (torch tensors; grads zero-initialized).

    placement = "plain" (the default): four ordinary allocations.

    placement = "spread" (opt-in; a benchmark's experiment, not something a caller of the C ABI gets):
    MI355X's 288 GiB are three physical ranges of 96 GiB (the three ranks of its 12-high HBM3E
    stacks).  The update streams through params, state0 and state1 in lockstep, and while all of them
    lie in one such range they compete for its banks: timed at K*P = 0.96e9, the same kernel runs at
    5.6-5.9 TB/s with the arrays adjacent and at 6.4-6.5 TB/s with at least one of them in another
    range (single-array kernels do not care).  Physical addresses cannot be asked for, but
    equal-sized allocations made in a row are handed out in physical order, cyclically from wherever
    the driver's free list happens to start: so nearly all free memory is taken in chunks of one
    array's size, the arrays are the chunks at 0, 1/3 and 2/3 of that sequence (which cannot all
    share a range, whatever the starting point), and the other chunks are given back at once.  It
    relies on undocumented allocator behaviour, needs most of the memory free (it falls back to
    the plain allocation when a chunk cannot be had) and only applies to arrays of at least 512 MiB
    that would all fit one range.
    """
    f32 = dict(dtype=torch.float32, device=dev)
    n = K * P * 4

    def plain():
        params = torch.empty((K, P), **f32)
        grads = torch.zeros((K, P), **f32)
        state0 = torch.empty((K, P), **f32)
        state1 = torch.empty((K, P), **f32) if second_moment else None
        return params, grads, state0, state1, "plain"

    if placement not in ("plain", "spread"):
        raise ValueError("placement: 'plain' or 'spread'")
    m = 0
    if placement == "spread":
        free, total = torch.cuda.mem_get_info(dev)
        if n >= (512 << 20) and 4 * n <= total // 3:
            m = int((free - (8 << 30)) // (n + (2 << 20)))
    if m < 12:
        return plain()
    chunks = []
    try:
        for _ in range(m):
            chunks.append(torch.empty((K, P), **f32))
    except RuntimeError:                   # someone else holds memory: give everything back
        del chunks
        torch.cuda.empty_cache()
        return plain()
    # The averaging streams through the K rows of params alone; it gains the same way when that one
    # array straddles the border between two ranges (5.6 -> 6.3 TB/s), which two or three chunks of
    # the sequence do.  They are found by timing the averaging itself on every chunk.
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def averaging_ms(c):
        best = float("inf")
        for rep in range(3):               # the first pass also warms up
            ev[0].record()
            average_rows(c)
            ev[1].record()
            ev[1].synchronize()
            if rep:
                best = min(best, ev[0].elapsed_time(ev[1]))
        return best

    with torch.cuda.device(dev):
        for c in chunks:
            c.zero_()                      # uninitialized memory may hold NaNs; not wanted even in a probe
        i0 = min(range(m), key=lambda i: averaging_ms(chunks[i]))
    at = lambda k: chunks[(i0 + k) % m]
    params, grads = at(0), at(1)
    if second_moment:
        state0, state1 = at(m // 3), at((2 * m) // 3)
    else:
        state0, state1 = at(m // 2), None
    grads.zero_()
    del chunks
    torch.cuda.empty_cache()
    return params, grads, state0, state1, "spread"


class Context:
    """Owns the device buffers (torch tensors) and a qsr_ctx.  Methods map 1:1 to the C ABI."""

    def __init__(self, w, theta0=None, model_const=None, eta_table=None, device="cuda:0", buffers=None,
                 placement="plain"):
        import torch
        self.torch = torch
        self.w = dict(w)
        self.dev = torch.device(device)
        K, P = w["K"], w["P"]
        with torch.cuda.device(self.dev):
            self.stream = torch.cuda.current_stream()
            cfg, self._keep = make_config(w, self.stream.cuda_stream, eta_table)
            self.cfg = cfg
            f32 = dict(dtype=torch.float32, device=self.dev)
            if buffers is not None:
                self.params, self.grads, self.state0, self.state1 = buffers
                self.placement = "caller"
            else:
                self.params, self.grads, self.state0, self.state1, self.placement = _allocate_state(
                    torch, self.dev, K, P, w["opt"] == "adamw", placement)
            self._theta0 = None if theta0 is None else torch.as_tensor(
                np.ascontiguousarray(theta0, dtype=np.float32)).to(self.dev)
            if theta0 is None:
                self.params.zero_()
            self.model_const = None if model_const is None else torch.as_tensor(
                np.ascontiguousarray(model_const, dtype=np.float32)).to(self.dev)
            nbytes = workspace_bytes(cfg)
            self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.dev)
            self._ctx = C.c_void_p()
            ptr = lambda t: C.c_void_p(0 if t is None else t.data_ptr())
            _check(lib().qsr_init(C.byref(cfg), ptr(self.params), ptr(self.grads), ptr(self.state0),
                                  ptr(self.state1), ptr(self._theta0), ptr(self.model_const),
                                  ptr(self.workspace), C.c_size_t(nbytes), C.byref(self._ctx)),
                   "qsr_init")

    # ---- the four calls of the hot path
    def local_step(self):
        _check(lib().qsr_local_step(self._ctx), "qsr_local_step")

    def maybe_sync(self):
        _check(lib().qsr_maybe_sync(self._ctx), "qsr_maybe_sync")

    def get_H(self):
        H, s, t = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib().qsr_get_H(self._ctx, C.byref(H), C.byref(s), C.byref(t)), "qsr_get_H")
        return H.value, s.value, t.value

    def step(self, n=1):
        L, ctx = lib(), self._ctx
        for _ in range(n):
            _check(L.qsr_local_step(ctx), "qsr_local_step")
            _check(L.qsr_maybe_sync(ctx), "qsr_maybe_sync")

    def run(self, n):
        """n iterations in one call; replays a captured HIP graph when the context was made on a
        stream other than the null stream (`with torch.cuda.stream(s): Context(...)`)."""
        _check(lib().qsr_run(self._ctx, C.c_int64(n)), "qsr_run")

    # ---- the rest of the ABI
    def read_sync_log(self):
        n = C.c_int64()
        _check(lib().qsr_read_sync_log(self._ctx, None, None, C.c_int64(0), C.byref(n)), "qsr_read_sync_log")
        t = np.zeros(max(n.value, 1), dtype=np.int64); H = np.zeros_like(t)
        _check(lib().qsr_read_sync_log(self._ctx, t.ctypes.data_as(C.c_void_p),
                                       H.ctypes.data_as(C.c_void_p), C.c_int64(n.value), C.byref(n)),
               "qsr_read_sync_log")
        return t[:n.value], H[:n.value]

    def read_host_schedule(self):
        """The rounds counted by the host's mirror of the schedule, as read_sync_log returns them."""
        n = C.c_int64()
        _check(lib().qsr_read_host_schedule(self._ctx, None, None, C.c_int64(0), C.byref(n)), "qsr_read_host_schedule")
        t = np.zeros(max(n.value, 1), dtype=np.int64); H = np.zeros_like(t)
        _check(lib().qsr_read_host_schedule(self._ctx, t.ctypes.data_as(C.c_void_p),
                                            H.ctypes.data_as(C.c_void_p), C.c_int64(n.value), C.byref(n)),
               "qsr_read_host_schedule")
        return t[:n.value], H[:n.value]

    def eta_table(self):
        eta = np.empty(self.w["T"], dtype=np.float64)
        _check(lib().qsr_eta_table(self._ctx, eta.ctypes.data_as(C.c_void_p), C.c_int64(len(eta))),
               "qsr_eta_table")
        return eta

    def read_loss(self):
        out = np.empty(self.w["K"], dtype=np.float32)
        _check(lib().qsr_read_loss(self._ctx, out.ctypes.data_as(C.c_void_p)), "qsr_read_loss")
        return out

    def get_state(self):
        st = (C.c_int64 * 4)()
        _check(lib().qsr_get_state(self._ctx, st), "qsr_get_state")
        return tuple(st)

    def set_state(self, state):
        st = (C.c_int64 * 4)(*state)
        _check(lib().qsr_set_state(self._ctx, st), "qsr_set_state")

    def restart(self):
        _check(lib().qsr_restart(self._ctx), "qsr_restart")

    def timing(self, on):
        _check(lib().qsr_timing(self._ctx, C.c_int(1 if on else 0)), "qsr_timing")

    def read_timing(self):
        ms = (C.c_double * 4)(); cnt = (C.c_int64 * 4)()
        _check(lib().qsr_read_timing(self._ctx, ms, cnt), "qsr_read_timing")
        return list(ms), list(cnt)

    def read_timing_stats(self):
        """(sum ms, count, min ms, median ms) per kind of bracket since the last read."""
        ms = (C.c_double * 4)(); cnt = (C.c_int64 * 4)(); lo = (C.c_double * 4)(); med = (C.c_double * 4)()
        _check(lib().qsr_read_timing_stats(self._ctx, ms, cnt, lo, med), "qsr_read_timing_stats")
        return list(ms), list(cnt), list(lo), list(med)

    def close(self):
        if self._ctx:
            lib().qsr_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
