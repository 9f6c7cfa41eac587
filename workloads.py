"""Named synthetic workloads and their seeded fixed inputs.

This module serves both the GPU library's callers and the CPU oracle's
callers.  It holds no arithmetic of the method: only the hyper-parameters of
each workload and the seeded draws of the *fixed* inputs (initial parameters,
the regression target w*, class means, the teacher map).  Per-iteration data
are drawn inside each implementation from Philox4x32-10, keyed
(seed; group, stream, worker, iteration).

The six workloads stand in for the paper's ImageNet runs (Sec. 4, App. C of
arXiv 2310.14423), which need a dataset and trained models that are not
available: "lsq" and "mlp" carry the ResNet recipe's optimizer (SGD, momentum
0.9, step or cosine decay), "flat60m"/"flat350m" carry the ViT recipe's
AdamW traffic at two sizes, "resmlp" has ViT-B's MLP sub-block shapes and
"vit" adds the attention sub-blocks (ViT-B's whole encoder block).
"""
import numpy as np


def _rng(seed, tag):
    return np.random.Generator(np.random.PCG64([int(seed), int(tag)]))


def mlp2_param_count(d_in, d_hidden, d_out):
    return d_in * d_hidden + d_hidden + d_hidden * d_out + d_out


def resmlp_param_count(d, d_hidden, n_blocks, n_heads=0):
    attn = 2 * d + d * 3 * d + 3 * d + d * d + d if n_heads else 0
    return n_blocks * (attn + 2 * d + d * d_hidden + d_hidden + d_hidden * d + d)


WORKLOADS = {
    # linear least squares, d=1024
    "lsq": dict(model="linreg", K=4, P=1024, T=256, T_warm=0, B_loc=32, d_in=1024,
                opt="sgdm", mu=0.9, lam=0.0, lr="cosine", eta_max=0.1, eta_min=0.0,
                H_base=2, alpha=0.2, data_sigma=0.1, seed=0),
    # two-layer perceptron 784-1024-10 on a 10-class Gaussian mixture
    "mlp": dict(model="mlp2", K=8, P=mlp2_param_count(784, 1024, 10), T=2000, T_warm=0,
                B_loc=128, d_in=784, d_hidden=1024, d_out=10,
                opt="sgdm", mu=0.9, lam=5e-4, lr="step", eta_max=0.8,
                milestones=(1000, 1500), factor=10.0,
                H_base=4, alpha=0.25, data_sigma=1.0, seed=0),
    # optimizer-only, 60 M parameters, 16 replicas
    "flat60m": dict(model="noise", K=16, P=60_000_000, T=5000, T_warm=0,
                    opt="adamw", beta1=0.9, beta2=0.999, eps=1e-8, lam=0.05,
                    lr="cosine", eta_max=1e-3, eta_min=0.0,
                    H_base=4, alpha=0.0175, grad_sigma=1e-3, seed=0),
    # 12 pre-LN residual MLP blocks, width 768 / 3072, 64 x 197 tokens per worker
    "resmlp": dict(model="resmlp", K=8, P=resmlp_param_count(768, 3072, 12), T=2000, T_warm=100,
                   B_loc=64 * 197, d_in=768, d_hidden=3072, n_blocks=12,
                   opt="adamw", beta1=0.9, beta2=0.999, eps=1e-8, lam=0.05,
                   lr="cosine", eta_max=8e-4, eta_min=0.0,
                   H_base=4, alpha=0.0175, seed=0),
    # the same 12 blocks, each preceded by its attention sub-block (12 heads of width 64, sequences
    # of 197 tokens): a whole ViT-B encoder block
    "vit": dict(model="resmlp", K=8, P=resmlp_param_count(768, 3072, 12, 12), T=2000, T_warm=100,
                B_loc=64 * 197, d_in=768, d_hidden=3072, n_blocks=12, n_heads=12, seq_len=197,
                opt="adamw", beta1=0.9, beta2=0.999, eps=1e-8, lam=0.05,
                lr="cosine", eta_max=8e-4, eta_min=0.0,
                H_base=4, alpha=0.0175, seed=0),
    # optimizer-only, 350 M parameters, 32 replicas (~180 GB of state)
    "flat350m": dict(model="noise", K=32, P=350_000_000, T=2000, T_warm=0,
                     opt="adamw", beta1=0.9, beta2=0.999, eps=1e-8, lam=0.05,
                     lr="cosine", eta_max=6e-4, eta_min=0.0,
                     H_base=2, alpha=0.01, grad_sigma=1e-3, seed=0),
}


def get(name, **overrides):
    w = dict(WORKLOADS[name])
    w.update(overrides)
    if w["model"] == "mlp2":
        w["P"] = mlp2_param_count(w["d_in"], w["d_hidden"], w["d_out"])
    elif w["model"] == "resmlp":
        w["P"] = resmlp_param_count(w["d_in"], w["d_hidden"], w["n_blocks"], w.get("n_heads", 0))
    elif w["model"] == "linreg":
        w["P"] = w["d_in"]
    return w


def theta0(w):
    """Initial parameters, float32 [P]; every worker starts from them."""
    m, seed = w["model"], w["seed"]
    if m in ("noise", "linreg", "external"):
        return np.zeros(w["P"], dtype=np.float32)
    r = _rng(seed, 1)
    if m == "mlp2":
        di, dh, do = w["d_in"], w["d_hidden"], w["d_out"]
        parts = [r.standard_normal(di * dh) / np.sqrt(di), np.zeros(dh),
                 r.standard_normal(dh * do) / np.sqrt(dh), np.zeros(do)]
        return np.concatenate(parts).astype(np.float32)
    if m == "resmlp":
        d, dh, L = w["d_in"], w["d_hidden"], w["n_blocks"]
        parts = []
        for _ in range(L):
            if w.get("n_heads", 0):     # attention sub-block: LayerNorm, q|k|v and output projections
                parts += [np.ones(d), np.zeros(d), 0.02 * r.standard_normal(d * 3 * d), np.zeros(3 * d),
                          0.02 * r.standard_normal(d * d), np.zeros(d)]
            parts += [np.ones(d), np.zeros(d), 0.02 * r.standard_normal(d * dh), np.zeros(dh),
                      0.02 * r.standard_normal(dh * d), np.zeros(d)]
        return np.concatenate(parts).astype(np.float32)
    raise ValueError(m)


def model_const(w):
    """The fixed part of the data distribution, float32, or None."""
    m, seed = w["model"], w["seed"]
    r = _rng(seed, 2)
    if m == "linreg":       # w* ~ N(0, I/d)
        return (r.standard_normal(w["d_in"]) / np.sqrt(w["d_in"])).astype(np.float32)
    if m == "mlp2":         # class means ~ N(0, I), [classes][d_in]
        return r.standard_normal((w["d_out"], w["d_in"])).astype(np.float32)
    if m == "resmlp":       # teacher map ~ N(0, 1), [d][d]
        return r.standard_normal((w["d_in"], w["d_in"])).astype(np.float32)
    return None
