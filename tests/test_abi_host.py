"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad configurations before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2310_14423_amd as qsr
import workloads
from paper_2310_14423_amd.binding import make_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "qsr.h")).read()
    declared = set(re.findall(r"\b(qsr_[a-z_A-Z]+)\s*\(", hdr))
    assert declared == set(qsr.EXPORTS)
    L = C.CDLL(qsr.lib_path())
    for name in declared:
        assert hasattr(L, name), name


def test_strerror():
    L = qsr.lib()
    assert L.qsr_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -6, -7):
        assert len(L.qsr_strerror(code)) > 3
    assert L.qsr_strerror(-99) == b"unknown error"


@pytest.mark.parametrize("name", ["lsq", "mlp", "flat60m", "resmlp", "vit", "flat350m"])
def test_named_workloads_validate(name):
    cfg, keep = make_config(workloads.get(name))
    assert qsr.validate(cfg) == (0, "ok")
    assert qsr.workspace_bytes(cfg) >= 0


@pytest.mark.parametrize("field,value,why", [
    ("K", 0, "K"), ("P", 0, "P"), ("T", 0, "T"), ("T_warm", -1, "T_warm"), ("T_warm", 6000, "T_warm"),
    ("opt", 2, "opt"), ("model", 5, "model"), ("lr_kind", 5, "lr_kind"), ("H_base", 0, "H_base"),
    ("alpha", -0.1, "alpha"), ("alpha", float("nan"), "alpha"), ("eta_max", 0.0, "eta_max"),
    ("eta_min", 1.0, "eta_min"), ("beta2", 1.0, "beta1/beta2"), ("eps", 0.0, "eps"),
    ("weight_decay", -1.0, "weight_decay"), ("grad_sigma", -1.0, "grad_sigma"), ("average_state", 2, "average_state"), ("fuse_sync", 2, "fuse_sync"), ("n_heads", 1, "n_heads"), ("reserved", 1, "reserved"), ("fuse_gradient", 3, "fuse_gradient"), ("clip_norm", -1.0, "clip_norm"),
    ("power", -1, "power"), ("power", 9, "power"), ("parallel", 2, "parallel"),
    ("parallel", 1, "parallel needs H_base = 1, power = 0"), ("t_local_start", -5, "t_local_start"), ("t_swap_start", 9999, "t_swap_start"),
])
def test_bad_configurations_are_rejected(field, value, why):
    cfg, keep = make_config(workloads.get("flat60m"))
    setattr(cfg, field, value)
    rc, msg = qsr.validate(cfg)
    assert rc == -1 and msg == why
    n = C.c_size_t(7)
    assert qsr.lib().qsr_workspace_bytes(C.byref(cfg), C.byref(n)) == -1 and n.value == 0
    out = C.c_void_p(1)
    rc = qsr.lib().qsr_init(C.byref(cfg), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16),
                            None, None, None, C.c_size_t(0), C.byref(out))
    assert rc == -1 and not out.value


def test_model_shape_checks():
    cfg, _ = make_config(workloads.get("mlp"))
    cfg.P += 1
    assert qsr.validate(cfg)[0] == -1
    cfg, _ = make_config(workloads.get("lsq"))
    cfg.d_in = 1000
    assert qsr.validate(cfg)[0] == -1


def test_attention_shape_checks():
    """Heads are 64 wide, sequences have 1..224 tokens and divide the local batch; the parameter
    count includes the attention arrays."""
    ok = workloads.get("vit")
    assert qsr.validate(make_config(ok)[0]) == (0, "ok")
    for bad in (dict(n_heads=6), dict(seq_len=0), dict(seq_len=225), dict(seq_len=200), dict(n_heads=-1)):
        cfg, _ = make_config(dict(ok, **bad))
        assert qsr.validate(cfg)[0] == -1, bad
    cfg, _ = make_config(dict(ok, P=workloads.get("resmlp")["P"]))
    assert qsr.validate(cfg)[0] == -1
    # the workspace grows by the q|k|v, attention-output and split-reduction buffers
    assert qsr.workspace_bytes(make_config(ok)[0]) > qsr.workspace_bytes(make_config(workloads.get("resmlp"))[0])


def test_null_arguments():
    L = qsr.lib()
    assert L.qsr_validate(None, None) == -1
    assert L.qsr_local_step(None) == -1 and L.qsr_maybe_sync(None) == -1
    assert L.qsr_get_H(None, None, None, None) == -1
    assert L.qsr_destroy(None) == -1
    assert L.qsr_get_state(None, None) == -1 and L.qsr_set_state(None, None) == -1
    assert L.qsr_average_rows(None, 2, C.c_int64(8), None) == -1
    cfg, _ = make_config(workloads.get("flat60m"))
    out = C.c_void_p()
    # NULL / misaligned buffers, missing second moment for AdamW
    assert L.qsr_init(C.byref(cfg), None, C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), None, None, None,
                      C.c_size_t(0), C.byref(out)) == -1
    assert L.qsr_init(C.byref(cfg), C.c_void_p(20), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), None, None,
                      None, C.c_size_t(0), C.byref(out)) == -1
    assert L.qsr_init(C.byref(cfg), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), None, None, None, None,
                      C.c_size_t(0), C.byref(out)) == -1
    # model workloads need their workspace and constants
    cfg, keep = make_config(workloads.get("lsq"))
    assert L.qsr_init(C.byref(cfg), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), None, None, None, None,
                      C.c_size_t(0), C.byref(out)) == -1


# ---- the library's host-side schedule (the routine behind the context's mirror of the device scheduler)
def _schedule_workload(T, T_warm, lr, eta_max, eta_min, H_base, alpha, power=2, **kw):
    w = dict(model="noise", K=1, P=4, T=T, T_warm=T_warm, opt="sgdm", mu=0.0, lam=0.0, lr=lr, eta_max=eta_max,
             eta_min=eta_min, H_base=H_base, alpha=alpha, power=power, grad_sigma=0.0, seed=0)
    w.update(kw)
    return w


def _golden_rows():
    from test_oracle_schedule import _rows
    return _rows()


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r["id"])
def test_host_schedule_reproduces_the_printed_communication_volumes(row):
    """Every communication volume the paper prints (Tables 1-3, Sec. 4.1, Table 6(a)), from the
    library's own learning-rate tables and host-side rule, and the same integer sequence as the
    oracle's."""
    import oracle
    from test_oracle_schedule import N_IMAGENET, _table
    spe = N_IMAGENET // row["B"]
    T = row["epochs"] * spe
    extra = {}
    lr = row["sched"]
    if lr == "smith":
        lr, extra = "step", dict(milestones=[e * spe for e in (150, 180, 210, 240, 270)], factor=2.0)
    w = _schedule_workload(T, row["Tw"], lr, row["eta_max"], row["eta_min"], row["H_base"], row["coef"],
                           power=3 if row["rule"] == "cubic" else 2, **extra)
    cfg, keep = make_config(w)
    t, H = qsr.host_schedule(cfg)
    assert t[-1] == T and H.sum() == T
    assert abs(100.0 * len(H) / T - row["pct"]) <= 0.05 + 1e-9
    eta, Tw = _table(row)
    oH, ot = oracle.schedule(eta, Tw, row["H_base"], row["coef"], 3 if row["rule"] == "cubic" else 2)
    assert np.array_equal(H, oH) and np.array_equal(t, ot)


@pytest.mark.parametrize("name,rounds", [("lsq", 28), ("mlp", 307), ("flat60m", 8), ("resmlp", 3), ("vit", 3),
                                         ("flat350m", 4)])
def test_host_schedule_of_the_named_workloads(name, rounds):
    import oracle
    from util import eta_of
    w = workloads.get(name)
    cfg, keep = make_config(w)
    t, H = qsr.host_schedule(cfg)
    oH, ot = oracle.schedule(eta_of(w), w.get("T_warm", 0), w["H_base"], w["alpha"])
    assert len(t) == rounds and np.array_equal(H, oH) and np.array_equal(t, ot)


@pytest.mark.parametrize("kw", [dict(power=3, alpha=0.012), dict(power=1, alpha=0.03), dict(power=0, H_base=7),
                                dict(power=0, H_base=8, t_local_start=700), dict(t_local_start=300),
                                dict(power=0, t_swap_start=1500), dict(alpha=100.0), dict(T_warm=2000),
                                dict(H_base=5000), dict(alpha=0.0, H_base=1)])
def test_host_schedule_variants_and_degenerate_cases(kw):
    """The rule variants and the edge cases of the truncation and warm-up rules, against the oracle's Alg. 2
    driver (post-local, SWAP, constant H; alpha so large that H = T; a run that is all warm-up)."""
    from util import oracle_run
    base = dict(T=2000, T_warm=0, lr="cosine", eta_max=0.008, eta_min=0.0, H_base=4, alpha=0.0175)
    base.update(kw)
    w = _schedule_workload(**base)
    cfg, keep = make_config(w)
    t, H = qsr.host_schedule(cfg)
    orc = oracle_run(dict(w, model="external", K=1, P=1), theta0=np.zeros(1))
    orc.step(w["T"], ext_g=np.zeros((w["T"], 1, 1)))
    assert np.array_equal(t, orc.sync_log) and np.array_equal(H, orc.H_log) and t[-1] == w["T"]


def test_clip_factors_argument_checks():
    """Host-side checks of the stateless clipping entry point: nothing is launched on bad arguments."""
    L = qsr.lib()
    n = C.c_size_t(7)
    assert L.qsr_clip_workspace_bytes(C.c_int32(0), C.c_int64(10), C.byref(n)) == -1 and n.value == 0
    assert L.qsr_clip_workspace_bytes(C.c_int32(4), C.c_int64(0), C.byref(n)) == -1
    assert L.qsr_clip_workspace_bytes(C.c_int32(4), C.c_int64(100), C.byref(n)) == 0 and n.value == 4 * 8
    assert L.qsr_clip_workspace_bytes(C.c_int32(2), C.c_int64(60_000_000), C.byref(n)) == 0 and n.value == 2 * 1024 * 8
    p = C.c_void_p(4096)
    call = lambda g, K, P, c, ws, wsb, coef, norm: L.qsr_clip_factors(
        g, C.c_int32(K), C.c_int64(P), C.c_float(c), ws, C.c_size_t(wsb), coef, norm, None)
    assert call(None, 2, 8, 1.0, p, 64, p, p) == -1
    assert call(p, 0, 8, 1.0, p, 64, p, p) == -1
    assert call(p, 2, 0, 1.0, p, 64, p, p) == -1
    assert call(p, 2, 8, 0.0, p, 64, p, p) == -1
    assert call(p, 2, 8, float("inf"), p, 64, p, p) == -1
    assert call(p, 2, 8, 1.0, None, 64, p, p) == -1
    assert call(p, 2, 8, 1.0, C.c_void_p(4097), 64, p, p) == -1      # misaligned workspace
    assert call(p, 2, 8, 1.0, p, 8, p, p) == -4                       # workspace too small
    assert call(p, 2, 8, 1.0, p, 64, None, p) == -1
