"""Seeded synthetic weight generators shared by the tests, the smoke run and the benchmark.

This module holds NO arithmetic of the quantisation method: it only draws random numbers of the shapes and
distributions of the five workloads and rounds them to bfloat16.  Both the HIP library and the CPU oracle are fed
from here; neither is imported here.

The real networks the paper quantises (Llama-3.x, Qwen-2.5, Mistral weights) are not available, so each workload
stands in for them with the shape of the corresponding layers and a zero-mean, mostly Gaussian, partly
heavy-tailed value distribution (the paper's own modelling assumption).

All generators take a torch device; the same (seed, device type) always gives the same bits.  A test draws its
input once and hands the identical bits to both sides.
"""
import math

import numpy as np
import torch

LLAMA7B_BLOCK = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                 ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA70B_LAYER = [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
                  ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def gaussian_matrix(rows, cols, std, seed, device="cpu"):
    """rows x cols entries i.i.d. N(0, std^2), rounded to bfloat16 (workload 0: 1024 x 1024, std 0.02)."""
    g = _gen(seed, device)
    return (torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16)


def gaussian_blocks(n_blocks, block, seed, device="cpu"):
    """n_blocks x block entries i.i.d. N(0, 1) as bfloat16 (the paper's Monte-Carlo codebook design input)."""
    return gaussian_matrix(n_blocks, block, 1.0, seed, device)


def student_t_matrix(rows, cols, nu, std, row_sigma, seed, device="cpu", chunk_rows=1024):
    """rows x cols Student-t(nu) entries scaled to standard deviation `std`; each output row is additionally
    scaled by exp(row_sigma * z_r), z_r ~ N(0, 1).  t = z / sqrt(chi2_nu / nu), chi2 as a sum of nu squared normals.
    """
    g = _gen(seed, device)
    unit = std / math.sqrt(nu / (nu - 2.0))
    out = torch.empty(rows, cols, dtype=torch.bfloat16, device=device)
    row_scale = torch.exp(row_sigma * torch.randn(rows, generator=g, device=device, dtype=torch.float32))
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        z = torch.randn(r1 - r0, cols, generator=g, device=device, dtype=torch.float32)
        chi2 = torch.zeros_like(z)
        for _ in range(int(nu)):
            chi2 += torch.randn(r1 - r0, cols, generator=g, device=device, dtype=torch.float32) ** 2
        t = z / torch.sqrt(chi2 / nu)
        out[r0:r1] = (t * unit * row_scale[r0:r1, None]).to(torch.bfloat16)
    return out


def llama7b_block(seed, device="cpu", scale=1):
    """Workload 1: the seven weight matrices of one Llama-7B-shaped transformer block, Student-t (nu=5) with
    std 0.02 and log-normal(0, 0.3) per-row jitter.  `scale` > 1 divides every dimension (reduced test sizes).
    Returns a list of (name, bf16 tensor [out, in])."""
    mats = []
    for k, (name, r, c) in enumerate(LLAMA7B_BLOCK):
        mats.append((name, student_t_matrix(r // scale, c // scale, 5.0, 0.02, 0.3, seed * 16 + k, device)))
    return mats


def llama70b_layer(seed, device="cpu", scale=1):
    """Workload 4 (one of its 80 layers): Llama-70B-shaped matrices, Student-t (nu=4), std 0.015, no row jitter."""
    mats = []
    for k, (name, r, c) in enumerate(LLAMA70B_LAYER):
        mats.append((name, student_t_matrix(r // scale, c // scale, 4.0, 0.015, 0.0, seed * 16 + k, device)))
    return mats


def flatten(mats):
    """Concatenate matrices in row-major order into one flat bf16 tensor (rows are multiples of every block size,
    so no block straddles a row or a matrix)."""
    return torch.cat([m.reshape(-1) for _, m in mats])


def plant_outliers(w, seed, frac=0.001, hot_cols=8, lo=10.0, hi=40.0):
    """Workload 3: overwrite round(frac * R * C) entries of the bf16 matrix `w` (in place) with +-U(lo, hi) times
    the standard deviation of their row.  Most of them sit in `hot_cols` random input columns: as many as fit, at
    most 80 % of the total and at most 90 % of the hot columns' entries; the rest are spread uniformly.
    Returns the sorted flat indices (int64, on w's device) of the planted entries."""
    rows, cols = w.shape
    dev = w.device
    g = _gen(seed, dev)
    total = int(round(frac * rows * cols))
    n_hot = min(int(0.8 * total), int(0.9 * hot_cols * rows))
    cols_hot = torch.randperm(cols, generator=g, device=dev)[:hot_cols]
    slots = torch.randperm(hot_cols * rows, generator=g, device=dev)[:n_hot]
    flat_hot = (slots // hot_cols) * cols + cols_hot[slots % hot_cols]
    rest = total - n_hot
    flat_rest = torch.randint(0, rows * cols, (2 * rest + 16,), generator=g, device=dev)
    flat = torch.unique(torch.cat([flat_hot, flat_rest]))
    keep_hot = torch.isin(flat, flat_hot)
    others = flat[~keep_hot][torch.randperm(int((~keep_hot).sum()), generator=g, device=dev)[:rest]]
    flat = torch.sort(torch.cat([flat[keep_hot], others])).values
    row_std = w.float().std(dim=1)
    mag = lo + (hi - lo) * torch.rand(flat.numel(), generator=g, device=dev)
    sign = torch.where(torch.rand(flat.numel(), generator=g, device=dev) < 0.5, -1.0, 1.0)
    vals = (sign * mag * row_std[flat // cols]).to(torch.bfloat16)
    w.view(-1)[flat] = vals
    return flat


def bits(t):
    """bf16 tensor -> numpy uint16 bit patterns on the host (what the oracle consumes)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)
