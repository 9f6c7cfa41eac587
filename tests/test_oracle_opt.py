"""Pins of the oracle's optimizer steps, averaging and Alg. 2 driver
(arXiv 2310.14423, Sec. 2 and Alg. 2; OPT per App. C)."""
import numpy as np
import pytest
import torch

import oracle


def test_sgdm_unrolled_closed_form():
    # lambda = 0: theta_n = theta_0 - sum_t eta_t sum_{j<=t} mu^(t-j) g_j
    rng = np.random.default_rng(0)
    n, T, mu = 7, 12, 0.9
    th0 = rng.standard_normal(n)
    g = rng.standard_normal((T, n))
    eta = rng.uniform(0.01, 0.2, T)
    th, buf = th0.copy(), np.zeros(n)
    for t in range(T):
        oracle.sgdm_step(th, buf, g[t], eta[t], mu, 0.0)
    want = th0.copy()
    for t in range(T):
        want -= eta[t] * sum(mu ** (t - j) * g[j] for j in range(t + 1))
    assert np.allclose(th, want, rtol=1e-13, atol=1e-14)


def test_sgdm_first_step_with_weight_decay():
    th = np.array([2.0, -1.0]); buf = np.zeros(2)
    oracle.sgdm_step(th, buf, np.array([0.5, 0.25]), 0.1, 0.9, 0.01)
    # theta_1 = theta_0 - eta (g + lambda theta_0)
    assert np.allclose(th, [2.0 - 0.1 * (0.5 + 0.02), -1.0 - 0.1 * (0.25 - 0.01)], rtol=1e-15)
    assert np.allclose(buf, [0.52, 0.24], rtol=1e-15)


def test_adamw_first_step_closed_form():
    # zero state: mhat = g, vhat = g^2  =>  theta_1 = theta_0 (1 - eta lambda) - eta g/(|g|+eps)
    th0 = np.array([1.0, -2.0, 0.5]); g = np.array([0.3, -4.0, 1e-12])
    th, m, v = th0.copy(), np.zeros(3), np.zeros(3)
    eta, lam, eps = 1e-2, 0.05, 1e-8
    oracle.adamw_step(th, m, v, g, eta, 0.9, 0.999, eps, lam, 1)
    want = th0 * (1 - eta * lam) - eta * g / (np.abs(g) + eps)
    assert np.allclose(th, want, rtol=1e-12)
    assert np.allclose(m, 0.1 * g, rtol=1e-12) and np.allclose(v, 0.001 * g * g, rtol=1e-12)


def test_adamw_moments_are_exponential_averages():
    rng = np.random.default_rng(1)
    n, T, b1, b2 = 5, 30, 0.9, 0.99
    g = rng.standard_normal((T, n))
    th, m, v = np.zeros(n), np.zeros(n), np.zeros(n)
    for t in range(T):
        oracle.adamw_step(th, m, v, g[t], 1e-3, b1, b2, 1e-8, 0.0, t + 1)
    wm = (1 - b1) * sum(b1 ** (T - 1 - j) * g[j] for j in range(T))
    wv = (1 - b2) * sum(b2 ** (T - 1 - j) * g[j] ** 2 for j in range(T))
    assert np.allclose(m, wm, rtol=1e-12) and np.allclose(v, wv, rtol=1e-12)


@pytest.mark.parametrize("opt", ["sgdm", "adamw"])
def test_K1_run_equals_library_optimizer(opt):
    """K = 1: averaging is the identity and Local OPT is the serial optimizer;
    the serial optimizer is checked against the PyTorch one in double precision."""
    rng = np.random.default_rng(2)
    n, T = 11, 40
    eta = oracle.lr_cosine(T, 5, 0.05, 0.0)
    g = rng.standard_normal((T, 1, n))
    th0 = rng.standard_normal(n)
    kw = dict(mu=0.9, lam=0.01) if opt == "sgdm" else dict(beta1=0.9, beta2=0.95, eps=1e-8, lam=0.1)
    run = oracle.Run(K=1, n=n, eta=eta, T_warm=5, opt=opt, H_base=3, alpha=0.02, theta0=th0, **kw)
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    if opt == "sgdm":
        o = torch.optim.SGD([p], lr=1.0, momentum=0.9, weight_decay=0.01)
    else:
        o = torch.optim.AdamW([p], lr=1.0, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    for t in range(T):
        run.step(1, ext_g=g[t:t + 1])
        for grp in o.param_groups:
            grp["lr"] = float(eta[t])
        p.grad = torch.tensor(g[t, 0])
        o.step()
        assert np.allclose(run.theta[0], p.detach().numpy(), rtol=1e-11, atol=1e-13), t
    assert run.t == T and run.sync_log[-1] == T


def test_average_is_the_mean_written_to_all_rows():
    rng = np.random.default_rng(3)
    th = rng.standard_normal((5, 9))
    want = th.mean(axis=0)
    oracle.average(th)
    for k in range(5):
        assert np.allclose(th[k], want, rtol=1e-15)
        assert np.array_equal(th[k], th[0])
    before = th.copy()
    oracle.average(th)                     # idempotent up to rounding
    assert np.allclose(th, before, rtol=1e-15)


def _brute_local_opt(K, n, eta, Tw, Hb, alpha, g, th0, opt, hp):
    """Alg. 2 written again in plain NumPy (tiny sizes only)."""
    T = len(eta)
    th = np.tile(th0, (K, 1)); a = np.zeros((K, n)); b = np.zeros((K, n))
    t = 0; syncs = []; Hs = []
    while t < T:
        e = eta[max(t, Tw)]
        H = T - t
        if e > 0 and (alpha / e) ** 2 < T - t:
            H = min(max(Hb, int(np.floor((alpha / e) * (alpha / e)))), T - t)
        Hs.append(H)
        for h in range(H):
            for k in range(K):
                gk = g[t + h, k]
                if opt == "sgdm":
                    a[k] = hp["mu"] * a[k] + gk + hp["lam"] * th[k]
                    th[k] = th[k] - eta[t + h] * a[k]
                else:
                    nstep = t + h + 1
                    a[k] = hp["b1"] * a[k] + (1 - hp["b1"]) * gk
                    b[k] = hp["b2"] * b[k] + (1 - hp["b2"]) * gk * gk
                    mh = a[k] / (1 - hp["b1"] ** nstep); vh = b[k] / (1 - hp["b2"] ** nstep)
                    th[k] = th[k] * (1 - eta[t + h] * hp["lam"]) - eta[t + h] * mh / (np.sqrt(vh) + hp["eps"])
        th[:] = th.mean(axis=0)
        t += H
        syncs.append(t)
    return th, Hs, syncs


@pytest.mark.parametrize("opt", ["sgdm", "adamw"])
@pytest.mark.parametrize("K,n", [(1, 1), (2, 3), (3, 2)])
def test_driver_brute_force_tiny(opt, K, n):
    rng = np.random.default_rng(10 * K + n)
    T, Tw = 20, 3
    eta = oracle.lr_cosine(T, Tw, 0.3, 0.0)
    g = rng.standard_normal((T, K, n))
    th0 = rng.standard_normal(n)
    hp = dict(mu=0.8, lam=0.02, b1=0.9, b2=0.98, eps=1e-8)
    kw = dict(mu=0.8, lam=0.02) if opt == "sgdm" else dict(beta1=0.9, beta2=0.98, eps=1e-8, lam=0.02)
    run = oracle.Run(K=K, n=n, eta=eta, T_warm=Tw, opt=opt, H_base=2, alpha=0.6, theta0=th0, **kw)
    run.step(T, ext_g=g)
    want, Hs, syncs = _brute_local_opt(K, n, eta, Tw, 2, 0.6, g, th0, opt, hp)
    assert list(run.H_log) == Hs and list(run.sync_log) == syncs and len(Hs) > 2
    assert np.allclose(run.theta, want, rtol=1e-12, atol=1e-14)


def test_replicas_identical_after_every_sync_and_differ_between():
    rng = np.random.default_rng(4)
    K, n, T = 4, 6, 30
    eta = oracle.lr_cosine(T, 0, 0.1, 0.0)
    run = oracle.Run(K=K, n=n, eta=eta, opt="adamw", lam=0.01, H_base=3, alpha=0.25,
                     theta0=rng.standard_normal(n))
    for t in range(T):
        run.step(1, ext_g=rng.standard_normal((1, K, n)))
        same = all(np.array_equal(run.theta[k], run.theta[0]) for k in range(K))
        assert same == (run.state.h == 0)
    assert run.t == T and run.sync_log[-1] == T


def test_optimizer_state_stays_local_across_a_sync():
    K, n = 2, 3
    run = oracle.Run(K=K, n=n, eta=np.full(4, 0.1), opt="sgdm", mu=0.9, H_base=2, alpha=0.0)
    g = np.zeros((2, K, n)); g[:, 0] = 1.0; g[:, 1] = -3.0
    run.step(2, ext_g=g)
    assert run.rounds == 1
    assert np.allclose(run.st0[0], 1.9) and np.allclose(run.st0[1], -5.7)   # not averaged, not reset


def test_workers_are_independent_between_syncs():
    """Permuting the workers' gradient streams permutes the rows (no cross-talk before a sync)."""
    rng = np.random.default_rng(6)
    K, n = 3, 4
    eta = np.full(10, 0.05)
    g = rng.standard_normal((5, K, n))
    a = oracle.Run(K=K, n=n, eta=eta, opt="adamw", H_base=10, alpha=0.0)
    b = oracle.Run(K=K, n=n, eta=eta, opt="adamw", H_base=10, alpha=0.0)
    perm = [2, 0, 1]
    a.step(5, ext_g=g); b.step(5, ext_g=g[:, perm])
    assert np.array_equal(a.theta[perm], b.theta)


def test_step_past_T_is_an_error():
    run = oracle.Run(K=1, n=1, eta=np.full(2, 0.1))
    run.step(2, ext_g=np.zeros((2, 1, 1)))
    with pytest.raises(RuntimeError):
        run.step(1, ext_g=np.zeros((1, 1, 1)))


# ---------------------------------------------------------------------------------------------
# Parallel OPT (Alg. 1) and the other synchronization schedules the paper compares with
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("opt", ["sgdm", "adamw"])
def test_parallel_opt_is_the_serial_optimizer_on_the_mean_gradient(opt):
    rng = np.random.default_rng(11)
    K, n, T = 3, 5, 12
    eta = oracle.lr_cosine(T, 2, 0.05, 0.0)
    g = rng.standard_normal((T, K, n))
    th0 = rng.standard_normal(n)
    kw = dict(mu=0.9, lam=0.01) if opt == "sgdm" else dict(beta1=0.9, beta2=0.95, eps=1e-8, lam=0.1)
    run = oracle.Run(K=K, n=n, eta=eta, T_warm=2, opt=opt, H_base=1, alpha=0.0, power=0, parallel=True,
                     theta0=th0, **kw)
    run.step(T, ext_g=g)
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    o = (torch.optim.SGD([p], lr=1.0, momentum=0.9, weight_decay=0.01) if opt == "sgdm" else
         torch.optim.AdamW([p], lr=1.0, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1))
    for t in range(T):
        for grp in o.param_groups:
            grp["lr"] = float(eta[t])
        p.grad = torch.tensor(g[t].mean(axis=0))
        o.step()
    for k in range(K):
        assert np.allclose(run.theta[k], p.detach().numpy(), rtol=1e-11, atol=1e-13)
    assert run.rounds == T                     # every step communicates: volume 100 %


def test_parallel_sgd_equals_local_sgd_with_H1():
    """Sec. 3 of the paper: parallel SGD is Local SGD with H = 1 (also with momentum, since the
    update is linear in the gradient and every worker restarts from the same point)."""
    rng = np.random.default_rng(12)
    K, n, T = 4, 6, 15
    eta = oracle.lr_cosine(T, 0, 0.1, 0.0)
    g = rng.standard_normal((T, K, n))
    for mu in (0.0, 0.9):
        a = oracle.Run(K=K, n=n, eta=eta, opt="sgdm", mu=mu, H_base=1, alpha=0.0, parallel=True)
        b = oracle.Run(K=K, n=n, eta=eta, opt="sgdm", mu=mu, H_base=1, alpha=0.0)
        a.step(T, ext_g=g); b.step(T, ext_g=g)
        assert np.allclose(a.theta, b.theta, rtol=1e-12, atol=1e-14)


def test_post_local_and_constant_and_power_schedules():
    T = 60
    eta = oracle.lr_cosine(T, 0, 0.1, 0.0)
    g = np.zeros((T, 1, 1))
    # constant H (power 0): rounds of 7, last one cut
    r = oracle.Run(K=1, n=1, eta=eta, H_base=7, alpha=0.3, power=0)
    r.step(T, ext_g=g)
    assert list(r.H_log) == [7] * 8 + [4]
    # post-local: H = 1 for rounds starting before t = 20, then constant 8
    r = oracle.Run(K=1, n=1, eta=eta, H_base=8, alpha=0.0, power=0, t_local_start=20)
    r.step(T, ext_g=g)
    assert list(r.H_log) == [1] * 20 + [8] * 5
    # Local OPT + SWAP (App. G): constant 4 until t = 30, then local steps only and one last averaging
    r = oracle.Run(K=1, n=1, eta=eta, H_base=4, alpha=0.0, power=0, t_swap_start=30)
    r.step(T, ext_g=g)
    assert list(r.H_log) == [4] * 8 + [28] and list(r.sync_log)[-2:] == [32, 60]
    # H ~ 1/eta and the cubic rule follow the power form of Eq. (2)
    for gamma, coef in ((1, 0.9), (3, 0.12)):
        r = oracle.Run(K=1, n=1, eta=eta, H_base=2, alpha=coef, power=gamma)
        r.step(T, ext_g=g)
        H, st = oracle.schedule(eta, 0, 2, coef, gamma)
        assert list(r.H_log) == list(H) and list(r.sync_log) == list(st) and len(H) > 3
        t = 0
        for Hs in H:
            v = (coef / eta[t]) ** gamma if eta[t] > 0 else np.inf
            want = T - t if not v < T - t else min(max(2, int(np.floor(v + 1e-12))), T - t)
            if abs(v - round(v)) > 1e-6:
                assert Hs == want
            t += Hs


def test_state_averaging_option():
    """Alg. 2 averages the parameters only; with the option on, the optimizer state is averaged
    at each synchronization too (and otherwise nothing changes)."""
    rng = np.random.default_rng(13)
    K, n = 3, 4
    eta = np.full(6, 0.05)
    g = rng.standard_normal((6, K, n))
    a = oracle.Run(K=K, n=n, eta=eta, opt="adamw", lam=0.01, H_base=3, alpha=0.0, average_state=True)
    b = oracle.Run(K=K, n=n, eta=eta, opt="adamw", lam=0.01, H_base=3, alpha=0.0)
    a.step(2, ext_g=g[:2]); b.step(2, ext_g=g[:2])
    assert np.array_equal(a.theta, b.theta) and np.array_equal(a.st0, b.st0)      # before the first sync
    a.step(1, ext_g=g[2:3]); b.step(1, ext_g=g[2:3])
    assert np.array_equal(a.theta, b.theta)                                       # parameters agree at the sync
    for st_a, st_b in ((a.st0, b.st0), (a.st1, b.st1)):
        assert np.allclose(st_a, np.tile(st_b.mean(axis=0), (K, 1)), rtol=1e-15)
        assert not np.allclose(st_b[0], st_b[1])
    a.step(3, ext_g=g[3:]); b.step(3, ext_g=g[3:])
    assert not np.allclose(a.theta, b.theta)                                      # and the runs differ afterwards


def test_gradient_clipping_equals_the_library_routine():
    """App. C's gradient clipping (by global norm, per worker): the oracle's clipped run is the
    library's clip_grad_norm_ followed by the library's optimizer, in double precision; below
    the threshold nothing changes, far above it the gradient has the threshold's norm."""
    rng = np.random.default_rng(5)
    n, T, K = 13, 25, 2
    eta = oracle.lr_cosine(T, 3, 0.02, 0.0)
    g = rng.standard_normal((T, K, n)) * rng.choice([0.05, 1.0, 20.0], size=(T, 1, 1))
    th0 = rng.standard_normal(n)
    run = oracle.Run(K=K, n=n, eta=eta, T_warm=3, opt="adamw", beta1=0.9, beta2=0.95, eps=1e-8, lam=0.1,
                     H_base=T, alpha=0.0, theta0=th0, clip_norm=1.0)      # one round: workers stay apart
    ps = [torch.tensor(th0, dtype=torch.float64, requires_grad=True) for _ in range(K)]
    os_ = [torch.optim.AdamW([p], lr=1.0, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1) for p in ps]
    for t in range(T - 1):
        run.step(1, ext_g=g[t:t + 1])
        for k in range(K):
            os_[k].param_groups[0]["lr"] = float(eta[t])
            ps[k].grad = torch.tensor(g[t, k])
            torch.nn.utils.clip_grad_norm_([ps[k]], max_norm=1.0)
            os_[k].step()
            assert np.allclose(run.theta[k], ps[k].detach().numpy(), rtol=1e-11, atol=1e-13), (t, k)
    # the routine itself
    small = np.array([0.3, -0.4]); big = np.array([30.0, -40.0])
    a = small.copy(); oracle.clip(a, 1.0)
    assert np.array_equal(a, small)
    b = big.copy(); norm = oracle.clip(b, 1.0)
    assert norm == pytest.approx(50.0, rel=1e-15)
    assert np.linalg.norm(b) == pytest.approx(1.0, rel=1e-6) and np.allclose(b / np.linalg.norm(b), big / 50.0)
    # clipping changes the trajectory when gradients are large, and not otherwise
    free = oracle.Run(K=K, n=n, eta=eta, T_warm=3, opt="sgdm", mu=0.9, H_base=T, theta0=th0)
    clipped = oracle.Run(K=K, n=n, eta=eta, T_warm=3, opt="sgdm", mu=0.9, H_base=T, theta0=th0, clip_norm=1e9)
    free.step(5, ext_g=g[:5]); clipped.step(5, ext_g=g[:5])
    assert np.array_equal(free.theta, clipped.theta)
