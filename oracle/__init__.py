"""ctypes front end of the CPU oracle (oracle/*.c).

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this package; the GPU library never does, and
this package never imports the GPU library.

The C sources are compiled with gcc on first use into oracle/_build/.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, f) for f in ("qsr_oracle.c", "qsr_oracle_resmlp.c")]
_HDR = [os.path.join(_HERE, "qsr_oracle.h")]
_SO = os.path.join(_HERE, "_build", "libqsr_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle.  -ffp-contract=off: no fused multiply-adds, so that the
    arithmetic is exactly the one written in the source."""
    os.makedirs(os.path.dirname(_SO), exist_ok=True)
    newest = max(os.path.getmtime(p) for p in _SRC + _HDR)
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < newest:
        tmp = _SO + ".%d.tmp" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-Wextra", "-o", tmp] + _SRC + ["-lm"])
        os.replace(tmp, _SO)
        # the driver of the sanitizer test (tests/test_oracle_sanitize.py builds it again with the
        # sanitizers on): compiled here too, so that a build covers every C file of this package
        drv = os.path.join(_HERE, "sanitize_driver.c")
        exe = os.path.join(os.path.dirname(_SO), "sanitize_driver")
        subprocess.check_call(["gcc", "-O1", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-o",
                               exe + ".%d.tmp" % os.getpid(), drv] + _SRC + ["-lm"])
        os.replace(exe + ".%d.tmp" % os.getpid(), exe)
    return _SO


class Config(C.Structure):
    _fields_ = [
        ("K", C.c_int32), ("opt", C.c_int32), ("model", C.c_int32), ("H_base", C.c_int32),
        ("n_threads", C.c_int32), ("n_blocks", C.c_int32), ("power", C.c_int32), ("parallel", C.c_int32),
        ("average_state", C.c_int32), ("n_heads", C.c_int32),
        ("n", C.c_int64), ("T", C.c_int64), ("T_warm", C.c_int64), ("t_local_start", C.c_int64),
        ("t_swap_start", C.c_int64), ("B_loc", C.c_int64),
        ("d_in", C.c_int64), ("d_hidden", C.c_int64), ("d_out", C.c_int64), ("seq_len", C.c_int64),
        ("mu", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
        ("lam", C.c_double), ("alpha", C.c_double), ("grad_sigma", C.c_double),
        ("data_sigma", C.c_double), ("clip_norm", C.c_double),
        ("seed", C.c_uint64),
        ("model_const", C.c_void_p), ("p_idx", C.c_void_p),
    ]


class State(C.Structure):
    _fields_ = [("t", C.c_int64), ("s", C.c_int64), ("h", C.c_int64), ("H", C.c_int64)]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.qsro_get_H_power.restype = C.c_int64
        _lib.qsro_get_H.restype = C.c_int64
        _lib.qsro_schedule.restype = C.c_int64
        for f in ("qsro_grad_linreg", "qsro_grad_mlp2", "qsro_grad_resmlp", "qsro_clip"):
            getattr(_lib, f).restype = C.c_double
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ---------------------------------------------------------------- schedules
def lr_cosine(T, T_warm, eta_max, eta_min=0.0):
    eta = np.empty(T, dtype=np.float64)
    lib().qsro_lr_cosine(C.c_int64(T), C.c_int64(T_warm), C.c_double(eta_max),
                         C.c_double(eta_min), _p(eta))
    return eta


def lr_linear(T, T_warm, eta_max, eta_min=0.0):
    eta = np.empty(T, dtype=np.float64)
    lib().qsro_lr_linear(C.c_int64(T), C.c_int64(T_warm), C.c_double(eta_max),
                         C.c_double(eta_min), _p(eta))
    return eta


def lr_pow2cos(T, T_warm, eta_max, eta_min=0.0):
    eta = np.empty(T, dtype=np.float64)
    lib().qsro_lr_pow2cos(C.c_int64(T), C.c_int64(T_warm), C.c_double(eta_max),
                          C.c_double(eta_min), _p(eta))
    return eta


def lr_step(T, T_warm, eta_max, milestones, factor):
    eta = np.empty(T, dtype=np.float64)
    ms = np.ascontiguousarray(milestones, dtype=np.int64)
    lib().qsro_lr_step(C.c_int64(T), C.c_int64(T_warm), C.c_double(eta_max),
                       C.c_int32(len(ms)), _p(ms), C.c_double(factor), _p(eta))
    return eta


def get_H(eta, T_warm, t, H_base, alpha, gamma=2):
    eta = _f64(eta)
    return int(lib().qsro_get_H_power(_p(eta), C.c_int64(len(eta)), C.c_int64(T_warm),
                                      C.c_int64(t), C.c_int64(H_base), C.c_double(alpha),
                                      C.c_int32(gamma)))


def schedule(eta, T_warm, H_base, alpha, gamma=2):
    """(H per round, iteration count at each averaging) for the whole run."""
    eta = _f64(eta)
    T = len(eta)
    n = int(lib().qsro_schedule(_p(eta), C.c_int64(T), C.c_int64(T_warm), C.c_int64(H_base),
                                C.c_double(alpha), C.c_int32(gamma), None, None, C.c_int64(0)))
    H = np.empty(n, dtype=np.int64)
    st = np.empty(n, dtype=np.int64)
    lib().qsro_schedule(_p(eta), C.c_int64(T), C.c_int64(T_warm), C.c_int64(H_base),
                        C.c_double(alpha), C.c_int32(gamma), _p(H), _p(st), C.c_int64(n))
    return H, st


# ---------------------------------------------------------------- random draws
def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().qsro_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def normal4(seed, stream, k, t, group):
    z = np.empty(4, dtype=np.float32)
    lib().qsro_normal4(C.c_uint64(seed), C.c_uint32(stream), C.c_uint32(k), C.c_uint64(t),
                       C.c_uint64(group), _p(z))
    return z


# ---------------------------------------------------------------- optimizer steps
def sgdm_step(theta, buf, g, eta, mu, lam):
    lib().qsro_sgdm_step(_p(theta), _p(buf), _p(_f64(g)), C.c_int64(theta.size), C.c_double(eta),
                         C.c_double(mu), C.c_double(lam))


def adamw_step(theta, m, v, g, eta, b1, b2, eps, lam, step):
    lib().qsro_adamw_step(_p(theta), _p(m), _p(v), _p(_f64(g)), C.c_int64(theta.size),
                          C.c_double(eta), C.c_double(b1), C.c_double(b2), C.c_double(eps),
                          C.c_double(lam), C.c_int64(step))


def clip(g, max_norm):
    """Clips one worker's gradient in place; returns its norm before clipping."""
    assert g.dtype == np.float64 and g.flags.c_contiguous
    return lib().qsro_clip(_p(g), C.c_int64(g.size), C.c_double(max_norm))


def average(theta):
    K, n = theta.shape
    lib().qsro_average(_p(theta), C.c_int32(K), C.c_int64(n))


# ---------------------------------------------------------------- Alg. 2 runs
MODELS = {"external": 0, "noise": 1, "linreg": 2, "mlp2": 3, "resmlp": 4}
OPTS = {"sgdm": 0, "adamw": 1}


class Run:
    """One Local-OPT run (Alg. 2) held in double precision on the CPU."""

    def __init__(self, *, K, n, eta, T_warm=0, opt="sgdm", mu=0.0, beta1=0.9, beta2=0.999,
                 eps=1e-8, lam=0.0, H_base=1, alpha=0.0, model="external", seed=0,
                 grad_sigma=0.0, data_sigma=0.0, B_loc=0, d_in=0, d_hidden=0, d_out=0,
                 n_blocks=0, model_const=None, p_idx=None, theta0=None, n_threads=1, power=2,
                 parallel=False, t_local_start=0, average_state=False, t_swap_start=0, clip_norm=0.0,
                 n_heads=0, seq_len=0):
        self.eta = _f64(eta)
        self.K, self.n = int(K), int(n)
        self._const = None if model_const is None else np.ascontiguousarray(model_const, np.float32)
        self._pidx = None if p_idx is None else np.ascontiguousarray(p_idx, np.int64)
        if n_heads:
            assert d_in % n_heads == 0 and seq_len > 0 and B_loc % seq_len == 0
        self.cfg = Config(K=K, opt=OPTS[opt], model=MODELS[model], H_base=H_base,
                          n_threads=n_threads, n_blocks=n_blocks, power=power, parallel=int(parallel), average_state=int(average_state),
                          t_local_start=t_local_start, t_swap_start=t_swap_start, n=n, T=len(self.eta),
                          T_warm=T_warm, B_loc=B_loc, d_in=d_in, d_hidden=d_hidden, d_out=d_out,
                          n_heads=n_heads, seq_len=seq_len, mu=mu, beta1=beta1, beta2=beta2, eps=eps, lam=lam, alpha=alpha,
                          grad_sigma=grad_sigma, data_sigma=data_sigma, clip_norm=clip_norm, seed=seed,
                          model_const=_p(self._const), p_idx=_p(self._pidx))
        self.state = State(0, 0, 0, 0)
        self.theta = np.zeros((K, n), dtype=np.float64)
        if theta0 is not None:
            self.theta[:] = np.asarray(theta0, dtype=np.float64)[None, :]
        self.st0 = np.zeros((K, n), dtype=np.float64)
        self.st1 = np.zeros((K, n), dtype=np.float64)
        cap = len(self.eta) + 1
        self._H = np.zeros(cap, dtype=np.int64)
        self._sync = np.zeros(cap, dtype=np.int64)

    def step(self, n_steps=1, ext_g=None, want_loss=False):
        g = None
        if self.cfg.model == 0:
            g = _f64(ext_g)
            assert g.shape == (n_steps, self.K, self.n)
        loss = np.zeros((n_steps, self.K), dtype=np.float64) if want_loss else None
        rc = lib().qsro_run(C.byref(self.cfg), _p(self.eta), C.byref(self.state), _p(self.theta),
                            _p(self.st0), _p(self.st1), C.c_int64(n_steps), _p(g), _p(self._H),
                            _p(self._sync), C.c_int64(len(self._H)), _p(loss))
        if rc != 0:
            raise RuntimeError("oracle: step past T or bad model")
        return loss

    @property
    def t(self):
        return self.state.t

    @property
    def rounds(self):
        return self.state.s

    @property
    def H_log(self):
        n = self.state.s + (1 if self.state.H else 0)
        return self._H[:n].copy()

    @property
    def sync_log(self):
        return self._sync[:self.state.s].copy()

    # single gradients (for pins)
    def grad(self, k, t, theta_k=None):
        g = np.zeros(self.n, dtype=np.float64)
        m = self.cfg.model
        th = None if theta_k is None else _f64(theta_k)
        L = lib()
        if m == 1:
            L.qsro_grad_noise(C.byref(self.cfg), C.c_int32(k), C.c_int64(t), _p(g))
            return g, 0.0
        f = {2: L.qsro_grad_linreg, 3: L.qsro_grad_mlp2, 4: L.qsro_grad_resmlp}[m]
        loss = f(C.byref(self.cfg), C.c_int32(k), C.c_int64(t), _p(th), _p(g))
        return g, float(loss)

    def linreg_batch(self, k, t):
        B, d = self.cfg.B_loc, self.cfg.d_in
        X = np.empty((B, d)); y = np.empty(B)
        lib().qsro_linreg_batch(C.byref(self.cfg), C.c_int32(k), C.c_int64(t), _p(X), _p(y))
        return X, y

    def mlp2_batch(self, k, t):
        B, d = self.cfg.B_loc, self.cfg.d_in
        X = np.empty((B, d)); lab = np.empty(B, dtype=np.int32)
        lib().qsro_mlp2_batch(C.byref(self.cfg), C.c_int32(k), C.c_int64(t), _p(X), _p(lab))
        return X, lab

    def resmlp_batch(self, k, t):
        M, d = self.cfg.B_loc, self.cfg.d_in
        X = np.empty((M, d)); Y = np.empty((M, d))
        lib().qsro_resmlp_batch(C.byref(self.cfg), C.c_int32(k), C.c_int64(t), _p(X), _p(Y))
        return X, Y
