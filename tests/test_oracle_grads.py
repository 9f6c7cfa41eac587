"""Pins of the oracle's local gradients (Eq. (1) of arXiv 2310.14423) on the three
model workloads: library autograd in double precision, finite differences, and the
paper's remark (Sec. 3) that Local SGD with H = 1 is data-parallel (minibatch) SGD."""
import numpy as np
import pytest
import torch

import oracle
import workloads


def _fd(run, k, t, theta, idxs, h=1e-6):
    out = []
    for i in idxs:
        a = theta.copy(); a[i] += h
        b = theta.copy(); b[i] -= h
        out.append((run.grad(k, t, a)[1] - run.grad(k, t, b)[1]) / (2 * h))
    return np.array(out)


def _mk(name, **ov):
    w = workloads.get(name, **ov)
    eta = np.full(w["T"], 0.1)
    run = oracle.Run(K=w["K"], n=w["P"], eta=eta, opt=w["opt"], model=w["model"], seed=w["seed"],
                     B_loc=w["B_loc"], d_in=w["d_in"], d_hidden=w.get("d_hidden", 0),
                     d_out=w.get("d_out", 0), n_blocks=w.get("n_blocks", 0),
                     data_sigma=w.get("data_sigma", 0.0), model_const=workloads.model_const(w),
                     theta0=workloads.theta0(w), n_heads=w.get("n_heads", 0), seq_len=w.get("seq_len", 0))
    return w, run


def test_linreg_batch_and_gradient():
    w, run = _mk("lsq", d_in=37, B_loc=9, K=3, T=8)
    wstar = workloads.model_const(w).astype(np.float64)
    X, y = run.linreg_batch(2, 5)
    # y - X w* is the observation noise: N(0, 0.1^2)
    big, brun = _mk("lsq", d_in=8, B_loc=20000, K=1, T=2)
    Xb, yb = brun.linreg_batch(0, 0)
    res = yb - Xb @ workloads.model_const(big).astype(np.float64)
    assert abs(res.std() - 0.1) < 0.003 and abs(res.mean()) < 0.003
    assert abs(Xb.std() - 1) < 0.01
    rng = np.random.default_rng(0)
    th = rng.standard_normal(37)
    g, loss = run.grad(2, 5, th)
    r = X @ th - y
    assert np.allclose(g, X.T @ r / 9, rtol=1e-12)
    assert loss == pytest.approx(0.5 * np.mean(r * r), rel=1e-12)
    assert np.allclose(g[:6], _fd(run, 2, 5, th, range(6)), rtol=1e-6, atol=1e-8)
    # batches of different workers / iterations differ
    X2, _ = run.linreg_batch(1, 5)
    X3, _ = run.linreg_batch(2, 6)
    assert not np.allclose(X, X2) and not np.allclose(X, X3)
    del wstar


def test_mlp2_gradient_matches_autograd():
    w, run = _mk("mlp", d_in=13, d_hidden=17, d_out=5, B_loc=11, K=2, T=4)
    di, dh, do = 13, 17, 5
    rng = np.random.default_rng(1)
    th = workloads.theta0(w).astype(np.float64) + 0.1 * rng.standard_normal(w["P"])
    X, lab = run.mlp2_batch(1, 3)
    means = workloads.model_const(w)
    assert lab.min() >= 0 and lab.max() < do
    # inputs = class mean + unit noise
    assert abs((X - means[lab]).std() - 1.0) < 0.15
    g, loss = run.grad(1, 3, th)
    p = torch.tensor(th, requires_grad=True)
    W1 = p[:di * dh].view(di, dh); b1 = p[di * dh:di * dh + dh]
    o = di * dh + dh
    W2 = p[o:o + dh * do].view(dh, do); b2 = p[o + dh * do:]
    hid = torch.relu(torch.tensor(X) @ W1 + b1)
    L = torch.nn.functional.cross_entropy(hid @ W2 + b2, torch.tensor(lab, dtype=torch.long))
    L.backward()
    assert loss == pytest.approx(L.item(), rel=1e-12)
    assert np.allclose(g, p.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_mlp2_labels_are_uniform():
    w, run = _mk("mlp", d_in=2, d_hidden=2, d_out=10, B_loc=20000, K=1, T=2)
    _, lab = run.mlp2_batch(0, 0)
    cnt = np.bincount(lab, minlength=10)
    assert cnt.min() > 1800 and cnt.max() < 2200


def test_resmlp_gradient_matches_autograd():
    w, run = _mk("resmlp", d_in=12, d_hidden=20, n_blocks=3, B_loc=7, K=2, T=4)
    d, dh, L = 12, 20, 3
    rng = np.random.default_rng(2)
    th = workloads.theta0(w).astype(np.float64) + 0.05 * rng.standard_normal(w["P"])
    X, Y = run.resmlp_batch(1, 2)
    WT = workloads.model_const(w).astype(np.float64)
    assert np.allclose(Y, X @ WT / np.sqrt(d), rtol=1e-12)
    g, loss = run.grad(1, 2, th)
    p = torch.tensor(th, requires_grad=True)
    x = torch.tensor(X)
    per = 2 * d + d * dh + dh + dh * d + d
    for l in range(L):
        q = p[l * per:(l + 1) * per]
        gam, bet = q[:d], q[d:2 * d]
        o = 2 * d
        W1 = q[o:o + d * dh].view(d, dh); o += d * dh
        b1 = q[o:o + dh]; o += dh
        W2 = q[o:o + dh * d].view(dh, d); o += dh * d
        b2 = q[o:o + d]
        u = torch.nn.functional.layer_norm(x, (d,), gam, bet, eps=1e-5)
        x = x + torch.nn.functional.gelu(u @ W1 + b1) @ W2 + b2
    Lt = 0.5 * ((x - torch.tensor(Y)) ** 2).mean()
    Lt.backward()
    assert loss == pytest.approx(Lt.item(), rel=1e-12)
    assert np.allclose(g, p.grad.numpy(), rtol=1e-9, atol=1e-14)
    idx = [0, d + 1, 2 * d + 5, per - 1, per + 3, 2 * per + 2 * d + d * dh + 1]
    assert np.allclose(g[idx], _fd(run, 1, 2, th, idx), rtol=1e-5, atol=1e-9)


def _vit_torch_loss(p, X, Y, d, dh, L, heads, S, attention=torch.nn.functional.scaled_dot_product_attention):
    """The attention + MLP blocks from library routines (layer_norm, the library's attention, gelu);
    p is the packed parameter tensor."""
    per_a = 2 * d + d * 3 * d + 3 * d + d * d + d
    per = per_a + 2 * d + d * dh + dh + dh * d + d
    x = torch.tensor(X)
    M = x.shape[0]
    for l in range(L):
        q = p[l * per:(l + 1) * per]
        o = 0
        def take(n, *shape):
            nonlocal o
            v = q[o:o + n]; o += n
            return v.view(*shape) if shape else v
        ga, ba = take(d), take(d)
        Wqkv, bqkv = take(d * 3 * d, d, 3 * d), take(3 * d)
        Wo, bo = take(d * d, d, d), take(d)
        gm, bm = take(d), take(d)
        W1, b1 = take(d * dh, d, dh), take(dh)
        W2, b2 = take(dh * d, dh, d), take(d)
        u = torch.nn.functional.layer_norm(x, (d,), ga, ba, eps=1e-5)
        z = (u @ Wqkv + bqkv).view(M // S, S, 3, heads, d // heads)        # [seq][tok][q|k|v][head][dk]
        qh, kh, vh = (z[:, :, i].permute(0, 2, 1, 3) for i in range(3))    # [seq][head][tok][dk]
        att = attention(qh, kh, vh)                                        # softmax(q k^T / sqrt(dk)) v
        x = x + att.permute(0, 2, 1, 3).reshape(M, d) @ Wo + bo
        u = torch.nn.functional.layer_norm(x, (d,), gm, bm, eps=1e-5)
        x = x + torch.nn.functional.gelu(u @ W1 + b1) @ W2 + b2
    return 0.5 * ((x - torch.tensor(Y)) ** 2).mean()


def test_vit_block_gradient_matches_autograd_of_the_library_attention():
    d, dh, L, heads, S = 12, 20, 2, 3, 5
    w, run = _mk("vit", d_in=d, d_hidden=dh, n_blocks=L, n_heads=heads, seq_len=S, B_loc=3 * S, K=2, T=4)
    assert w["P"] == L * (2 * d + 3 * d * d + 3 * d + d * d + d + 2 * d + 2 * d * dh + dh + d)
    rng = np.random.default_rng(5)
    # large enough weights that the attention probabilities are far from uniform
    th = workloads.theta0(w).astype(np.float64) + 0.3 * rng.standard_normal(w["P"])
    X, Y = run.resmlp_batch(1, 2)
    g, loss = run.grad(1, 2, th)
    p = torch.tensor(th, requires_grad=True)
    Lt = _vit_torch_loss(p, X, Y, d, dh, L, heads, S)
    Lt.backward()
    assert loss == pytest.approx(Lt.item(), rel=1e-12)
    assert np.allclose(g, p.grad.numpy(), rtol=1e-9, atol=1e-13)
    per_a = 2 * d + d * 3 * d + 3 * d + d * d + d
    per = w["P"] // L
    idx = [0, d + 2, 2 * d + 7, 2 * d + d * 3 * d - 1, 2 * d + d * 3 * d + d + 1, per_a - d - 3, per_a - 1,
           per_a + 1, per + 2 * d + 2 * d + 5, per + per_a + 2 * d + 3]
    assert np.allclose(g[idx], _fd(run, 1, 2, th, idx), rtol=1e-5, atol=1e-9)


def test_attention_special_cases_with_closed_forms():
    """(a) Sequences of one token: the softmax is 1, so the sub-block is x + (u Wv + bv) Wo + bo.
    (b) Zero query weights and bias: every probability is 1/S, so each token receives the mean
    value vector of its sequence.  Both written out in NumPy and compared through the loss."""
    d, dh, heads = 8, 6, 2
    rng = np.random.default_rng(9)

    def ref_loss(w, th, X, Y, mix):
        per_a = 2 * d + d * 3 * d + 3 * d + d * d + d
        ga, ba = th[:d], th[d:2 * d]
        Wqkv = th[2 * d:2 * d + 3 * d * d].reshape(d, 3 * d); bqkv = th[2 * d + 3 * d * d:2 * d + 3 * d * d + 3 * d]
        Wo = th[per_a - d - d * d:per_a - d].reshape(d, d); bo = th[per_a - d:per_a]
        m = th[per_a:]
        gm, bm = m[:d], m[d:2 * d]
        W1 = m[2 * d:2 * d + d * dh].reshape(d, dh); b1 = m[2 * d + d * dh:2 * d + d * dh + dh]
        W2 = m[2 * d + d * dh + dh:2 * d + d * dh + dh + dh * d].reshape(dh, d); b2 = m[-d:]
        def ln(x, g_, b_):
            mu = x.mean(1, keepdims=True); var = ((x - mu) ** 2).mean(1, keepdims=True)
            return g_ * (x - mu) / np.sqrt(var + 1e-5) + b_
        u = ln(X, ga, ba)
        v = u @ Wqkv[:, 2 * d:] + bqkv[2 * d:]
        x = X + mix(v) @ Wo + bo
        h = ln(x, gm, bm) @ W1 + b1
        from scipy.special import erf
        x = x + (0.5 * h * (1 + erf(h / np.sqrt(2)))) @ W2 + b2
        return 0.5 * np.mean((x - Y) ** 2)

    # (a)
    w, run = _mk("vit", d_in=d, d_hidden=dh, n_blocks=1, n_heads=heads, seq_len=1, B_loc=6, K=1, T=2)
    th = workloads.theta0(w).astype(np.float64) + 0.3 * rng.standard_normal(w["P"])
    X, Y = run.resmlp_batch(0, 1)
    assert run.grad(0, 1, th)[1] == pytest.approx(ref_loss(w, th, X, Y, lambda v: v), rel=1e-12)
    # (b)
    S = 3
    w, run = _mk("vit", d_in=d, d_hidden=dh, n_blocks=1, n_heads=heads, seq_len=S, B_loc=2 * S, K=1, T=2)
    th = workloads.theta0(w).astype(np.float64) + 0.3 * rng.standard_normal(w["P"])
    th[2 * d:2 * d + 3 * d * d].reshape(d, 3 * d)[:, :d] = 0.0          # Wq
    th[2 * d + 3 * d * d:2 * d + 3 * d * d + d] = 0.0                   # bq
    X, Y = run.resmlp_batch(0, 1)
    mean_of_sequence = lambda v: np.repeat(v.reshape(-1, S, d).mean(1), S, axis=0)
    assert run.grad(0, 1, th)[1] == pytest.approx(ref_loss(w, th, X, Y, mean_of_sequence), rel=1e-12)


def test_attention_groups_tokens_by_sequence():
    """Attention acts within a sequence (seq_len consecutive token rows) and the loss is a mean over
    tokens: reordering whole sequences leaves the library model's parameter gradient unchanged,
    moving one token into another sequence changes it, and the oracle agrees with the former."""
    d, dh, heads, S = 8, 6, 2, 4
    w, run = _mk("vit", d_in=d, d_hidden=dh, n_blocks=1, n_heads=heads, seq_len=S, B_loc=3 * S, K=1, T=2)
    rng = np.random.default_rng(3)
    th = workloads.theta0(w).astype(np.float64) + 0.3 * rng.standard_normal(w["P"])
    X, Y = run.resmlp_batch(0, 0)
    p = torch.tensor(th, requires_grad=True)
    _vit_torch_loss(p, X, Y, d, dh, 1, heads, S).backward()
    g1 = p.grad.numpy().copy()
    perm = np.concatenate([np.arange(S) + S * s for s in (2, 0, 1)])
    p2 = torch.tensor(th, requires_grad=True)
    _vit_torch_loss(p2, X[perm], Y[perm], d, dh, 1, heads, S).backward()
    assert np.allclose(g1, p2.grad.numpy(), rtol=1e-10, atol=1e-15)
    # whereas moving one token into another sequence does change it (the oracle groups by rows)
    swap = np.arange(3 * S); swap[0], swap[S] = swap[S], swap[0]
    p3 = torch.tensor(th, requires_grad=True)
    _vit_torch_loss(p3, X[swap], Y[swap], d, dh, 1, heads, S).backward()
    assert not np.allclose(g1, p3.grad.numpy(), rtol=1e-6)
    g, _ = run.grad(0, 0, th)
    assert np.allclose(g, g1, rtol=1e-9, atol=1e-13)


def test_local_sgd_with_H1_is_minibatch_sgd():
    """H = 1, plain SGD: the averaged iterate equals SGD on the K*B_loc batch."""
    w = workloads.get("lsq", d_in=10, B_loc=4, K=3, T=6)
    eta = oracle.lr_cosine(6, 0, 0.1)
    run = oracle.Run(K=3, n=10, eta=eta, opt="sgdm", mu=0.0, lam=0.0, H_base=1, alpha=0.0,
                     model="linreg", B_loc=4, d_in=10, data_sigma=0.1, seed=1,
                     model_const=workloads.model_const(w))
    th = np.zeros(10)
    for t in range(6):
        Xs, ys = zip(*[run.linreg_batch(k, t) for k in range(3)])
        X = np.concatenate(Xs); y = np.concatenate(ys)
        th = th - eta[t] * X.T @ (X @ th - y) / 12
        run.step(1)
        assert np.allclose(run.theta[0], th, rtol=1e-12, atol=1e-15)
    assert list(run.sync_log) == [1, 2, 3, 4, 5, 6]


def test_lsq_run_reduces_the_error_at_a_stable_step_size():
    """Sanity of the least-squares workload at a step size inside the mean-square stability
    region of momentum SGD with fresh batches (roughly eta/(1-mu) * (1 + d/B_loc) < 2, i.e.
    eta < 0.006 for d = 1024, B_loc = 32, mu = 0.9): the iterate approaches w* and the loss
    approaches the noise floor sigma^2/2 = 0.005.  (At the workload's own eta_max = 0.1 the
    iteration is far outside that region and the iterates grow by many orders of magnitude;
    that run is a parity case, not a convergence case.)"""
    w = workloads.get("lsq")
    eta = oracle.lr_cosine(w["T"], 0, 0.003)
    run = oracle.Run(K=4, n=1024, eta=eta, opt="sgdm", mu=0.9, H_base=2, alpha=0.2, model="linreg",
                     B_loc=32, d_in=1024, data_sigma=0.1, seed=0,
                     model_const=workloads.model_const(w), n_threads=4)
    loss = run.step(256, want_loss=True)
    assert run.t == 256 and run.sync_log[-1] == 256
    wstar = workloads.model_const(w).astype(np.float64)
    err0 = np.sum(wstar**2)
    err = np.sum((run.theta[0] - wstar) ** 2)
    assert err < 0.02 * err0
    assert 0.004 < loss[-20:].mean() < 0.03
