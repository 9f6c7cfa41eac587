"""Helpers shared by the tests: build the oracle run and the GPU context of one workload
from the same dictionary, and compare parameters to the stated tolerance."""
import numpy as np

import oracle
import workloads


def eta_of(w):
    if w["lr"] == "cosine":
        return oracle.lr_cosine(w["T"], w.get("T_warm", 0), w["eta_max"], w.get("eta_min", 0.0))
    if w["lr"] == "step":
        return oracle.lr_step(w["T"], w.get("T_warm", 0), w["eta_max"], list(w["milestones"]), w["factor"])
    if w["lr"] == "linear":
        return oracle.lr_linear(w["T"], w.get("T_warm", 0), w["eta_max"], w.get("eta_min", 0.0))
    if w["lr"] == "pow2cos":
        return oracle.lr_pow2cos(w["T"], w.get("T_warm", 0), w["eta_max"], w.get("eta_min", 0.0))
    raise ValueError(w["lr"])


def oracle_run(w, p_idx=None, n_threads=8, theta0=None, eta=None):
    n = w["P"] if p_idx is None else len(p_idx)
    th0 = workloads.theta0(w) if theta0 is None else theta0
    if p_idx is not None:
        th0 = np.asarray(th0)[p_idx]
    return oracle.Run(K=w["K"], n=n, eta=eta_of(w) if eta is None else eta, T_warm=w.get("T_warm", 0),
                      opt=w["opt"], mu=w.get("mu", 0.0), beta1=w.get("beta1", 0.9),
                      beta2=w.get("beta2", 0.999), eps=w.get("eps", 1e-8), lam=w.get("lam", 0.0),
                      H_base=w["H_base"], alpha=w["alpha"], model=w["model"], seed=w.get("seed", 0),
                      grad_sigma=w.get("grad_sigma", 0.0), data_sigma=w.get("data_sigma", 0.0),
                      B_loc=w.get("B_loc", 0), d_in=w.get("d_in", 0), d_hidden=w.get("d_hidden", 0),
                      d_out=w.get("d_out", 0), n_blocks=w.get("n_blocks", 0),
                      model_const=workloads.model_const(w), p_idx=p_idx, theta0=th0,
                      n_threads=n_threads, power=w.get("power", 2), parallel=w.get("parallel", False),
                      t_local_start=w.get("t_local_start", 0), average_state=w.get("average_state", False), t_swap_start=w.get("t_swap_start", 0),
                      clip_norm=w.get("clip_norm", 0.0), n_heads=w.get("n_heads", 0),
                      seq_len=w.get("seq_len", 0))


def gpu_ctx(w, theta0=None, eta_table=None):
    import paper_2310_14423_amd as qsr
    th0 = workloads.theta0(w) if theta0 is None else theta0
    return qsr.Context(w, theta0=th0, model_const=workloads.model_const(w), eta_table=eta_table)


# fp32 tolerance of the parameter comparison: |gpu - oracle| <= RTOL * (|oracle| + rms(oracle)).
# The rms term is the absolute floor for parameters that pass close to zero: an fp32 state
# cannot track them to a relative 1e-5 of their own (tiny) value.
RTOL_F32 = 1e-5


def assert_params_close(gpu, orc, rtol=RTOL_F32, what="", tail=None, rms=None):
    """Every entry within rtol * (|oracle| + rms(oracle)).  tail = (fraction, factor): that fraction
    of the entries may exceed the bound, none by more than the factor (for groups of millions of
    bf16 dot products, where the bound is about five standard deviations of the rounding noise).
    rms, if given, replaces rms(oracle) (for a group whose exact value is zero)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    orc = np.asarray(orc, dtype=np.float64)
    assert gpu.shape == orc.shape
    assert np.all(np.isfinite(gpu)), what
    if rms is None:
        rms = np.sqrt(np.mean(orc * orc))
    err = np.abs(gpu - orc)
    bound = rtol * (np.abs(orc) + rms)
    ratio = err / np.maximum(bound, 1e-300)
    msg = "%s: max |diff| %.3e, max ratio to bound %.3f (rms %.3e)" % (what, err.max(), ratio.max(), rms)
    if tail is None:
        assert ratio.max() <= 1.0, msg
    else:
        frac, factor = tail
        assert ratio.max() <= factor and np.count_nonzero(ratio > 1.0) <= np.ceil(frac * ratio.size), msg
    return float(np.max(err / np.maximum(bound, 1e-300)))


def rms_error_ratio(gpu, orc, rms=None):
    """rms(gpu - oracle) / rms(oracle) of one group (rms, if given, replaces rms(oracle))."""
    gpu = np.asarray(gpu, dtype=np.float64)
    orc = np.asarray(orc, dtype=np.float64)
    if rms is None:
        rms = np.sqrt(np.mean(orc * orc))
    err = gpu - orc
    return float(np.sqrt(np.mean(err * err)) / max(rms, 1e-300))


def assert_mirror_matches_device(ctx):
    """The rounds counted by the host's mirror of the schedule (which decides where an averaging kernel is
    enqueued) equal the device scheduler's log, entry for entry."""
    dt, dH = ctx.read_sync_log()
    mt, mH = ctx.read_host_schedule()
    assert list(dt) == list(mt) and list(dH) == list(mH), (list(dt), list(mt))
