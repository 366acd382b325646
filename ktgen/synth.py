"""Synthetic activation / rotation generators (no method arithmetic here)."""
import math

import numpy as np
import torch

# The five workloads; sizes and outlier recipes as named by the benchmark
# definition.  "steps"/"lr" describe how the workload is driven, not how X is made.
CONFIGS = {
    "C1": dict(n=2048, d=256, batch=1, dtype="f32", base="normal", outlier_cols=4,
               outlier_scale=50.0, t_frac=0.05, t_df=3, t_scale=10.0, R0="orthogonal",
               steps=1, lr=1e-2),
    "C2": dict(n=65536, d=2048, batch=1, dtype="bf16", base="normal", outlier_cols=16,
               outlier_scale=100.0, t_frac=0.05, t_df=3, t_scale=10.0, R0="identity",
               steps=10, lr=1e-2),
    "C3": dict(n=131072, d=4096, batch=1, dtype="bf16", base="normal", outlier_cols=32,
               outlier_scale="lognormal2", t_frac=0.0, t_df=3, t_scale=10.0,
               R0="orthogonal", steps=1, lr=1e-2),
    "C4": dict(n=131072, d=128, batch=256, dtype="bf16", base="t4", outlier_cols=2,
               outlier_scale=50.0, t_frac=0.0, t_df=3, t_scale=10.0, R0="orthogonal",
               steps=1, lr=1e-2),
    "C5": dict(n=1048576, d=8192, batch=1, dtype="bf16", base="normal", outlier_cols=64,
               outlier_scale=200.0, t_frac=0.05, t_df=3, t_scale=10.0, R0="orthogonal",
               steps=20, lr=1e-2),
}


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _student_t(shape, df, g, device):
    z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    chi = torch.zeros(shape, device=device, dtype=torch.float32)
    for _ in range(int(df)):
        chi += torch.randn(shape, generator=g, device=device, dtype=torch.float32) ** 2
    return z / torch.sqrt(chi / float(df))


def make_x(n, d, *, seed=0, base="normal", outlier_cols=0, outlier_scale=1.0,
           t_frac=0.0, t_df=3, t_scale=10.0, dtype="bf16", device="cpu",
           chunk_rows=8192):
    """Activations [n][d].

    Recipe, in this order: bulk entries N(0,1) (or Student-t(4) for ``base='t4'``);
    ``outlier_cols`` distinct random columns multiplied by ``outlier_scale`` (a
    float, or ``'lognormal2'`` for per-column factors exp(2 z), z ~ N(0,1)); then an
    i.i.d. Bernoulli(``t_frac``) mask of entries overwritten by ``t_scale`` times a
    Student-t(``t_df``) draw.  Returned in ``dtype`` ('bf16' or 'f32').
    """
    device = torch.device(device)
    g = _gen(seed, device)
    gc = _gen(seed + 7919, "cpu")
    cols = torch.randperm(d, generator=gc)[:outlier_cols]
    if outlier_scale == "lognormal2":
        fac = torch.exp(2.0 * torch.randn(outlier_cols, generator=gc))
    else:
        fac = torch.full((outlier_cols,), float(outlier_scale))
    colscale = torch.ones(d)
    colscale[cols] = fac
    colscale = colscale.to(device)
    out_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    X = torch.empty((n, d), dtype=out_dtype, device=device)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        shp = (r1 - r0, d)
        if base == "t4":
            blk = _student_t(shp, 4, g, device)
        else:
            blk = torch.randn(shp, generator=g, device=device, dtype=torch.float32)
        blk *= colscale
        if t_frac > 0.0:
            mask = torch.rand(shp, generator=g, device=device) < t_frac
            spikes = t_scale * _student_t(shp, t_df, g, device)
            blk = torch.where(mask, spikes, blk)
        X[r0:r1] = blk.to(out_dtype)
    return X


def random_orthogonal(d, seed=0, device="cpu"):
    """Haar-like orthogonal matrix: Q of a Gaussian's QR, columns sign-fixed by diag(R)."""
    g = _gen(seed + 104729, "cpu")
    a = torch.randn((d, d), generator=g, dtype=torch.float64)
    q, r = torch.linalg.qr(a)
    q = q * torch.sign(torch.diagonal(r)).unsqueeze(0)
    return q.to(torch.float32).contiguous().to(device)


def make_problem(name, *, seed=0, device="cpu", n=None, batch=None):
    """X (and R0 as fp32) for one of CONFIGS; ``n``/``batch`` may be overridden to take a
    smaller instance with the same recipe.  Returns (X [batch][n][d], R [batch][d][d], cfg)."""
    cfg = dict(CONFIGS[name])
    if n is not None:
        cfg["n"] = int(n)
    if batch is not None:
        cfg["batch"] = int(batch)
    xs, rs = [], []
    for b in range(cfg["batch"]):
        xs.append(make_x(cfg["n"], cfg["d"], seed=seed + 1000 * b, base=cfg["base"],
                         outlier_cols=cfg["outlier_cols"], outlier_scale=cfg["outlier_scale"],
                         t_frac=cfg["t_frac"], t_df=cfg["t_df"], t_scale=cfg["t_scale"],
                         dtype=cfg["dtype"], device=device))
        if cfg["R0"] == "identity":
            rs.append(torch.eye(cfg["d"], dtype=torch.float32, device=device))
        else:
            rs.append(random_orthogonal(cfg["d"], seed=seed + 1000 * b, device=device))
    return torch.stack(xs), torch.stack(rs), cfg


def bf16_round(t):
    """Round-to-nearest-even to bf16, returned as fp32 (the values a bf16 GEMM sees)."""
    return t.to(torch.bfloat16).to(torch.float32)


def to_f64(t):
    """Exact widening of a (bf16/fp32) tensor to a float64 numpy array on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()
