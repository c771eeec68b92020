"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves the tests (oracle side and GPU side alike) and the
benchmark.  It holds none of the method's arithmetic: it draws random
tensors, scales outlier channels, and hands out raw bits.  The fp32 -> bf16
conversion of generated data is torch's own `.to(torch.bfloat16)`.

Recipe (the paper trains LLaMA-family models with block size 128; these
tensors take the shapes of its GEMM operands and stand in for real
activations and gradients, which need the paper's datasets and weights):

* activation [rows, cols]: i.i.d. N(0,1) or Student-t(3) values; a fixed
  fraction of the columns ("outlier channels", chosen without replacement)
  is multiplied by a constant for every row; stored as bf16.
* gradient [n]: i.i.d. N(0, sigma^2) fp32 values; an i.i.d. Bernoulli mask
  multiplies a small fraction of the elements by a spike factor.

Host generators use numpy's PCG64; device generators use a seeded
torch.Generator on the GPU (same recipe, different stream of numbers) so
that multi-gigabyte benchmark inputs need no host round trip.
"""
import numpy as np

# ---- the five benchmark configurations ------------------------------------

HIDDEN_8B, FFN_8B = 4096, 14336
HIDDEN_32B, FFN_32B = 5120, 27648
# one LLaMA-8B decoder layer: q, o (4096x4096), k, v (4096x1024), gate, up, down (4096x14336)
LAYER_PARAMS_8B = 2 * 4096 * 4096 + 2 * 4096 * 1024 + 3 * 4096 * 14336

CONFIGS = {
    "tiny": dict(
        seed=0,
        act=dict(rows=256, cols=512, dist="normal", outlier_channels=4, outlier_scale=20.0),
        bits=4, group=128,
        grad=dict(n=1 << 20, sigma=1e-3, spike_frac=0.0, spike_scale=1.0, seeds=(1, 2, 3, 4)),
        K=4),
    "llama8b_act": dict(
        seed=10,
        acts=dict(A=dict(rows=4096, cols=HIDDEN_8B), F=dict(rows=4096, cols=FFN_8B)),
        dist="normal", outlier_frac=0.005, outlier_scale=30.0, group=128),
    "llama8b_grad": dict(
        seed=20, n=LAYER_PARAMS_8B, sigma=1e-4, spike_frac=0.001, spike_scale=100.0,
        K=8, group=128),
    "llama32b_act": dict(
        seed=30,
        acts=dict(A=dict(rows=4096, cols=HIDDEN_32B), F=dict(rows=4096, cols=FFN_32B)),
        dist="student_t3", outlier_frac=0.01, outlier_scale=50.0, groups=(64, 128)),
    "stage_sweep": dict(
        seed=40, rows=8192, hidden=HIDDEN_8B, ffn=FFN_8B, dist="normal",
        outlier_frac=0.005, outlier_scale=30.0, group=128,
        grad=dict(n=LAYER_PARAMS_8B, sigma=1e-4, spike_frac=0.001, spike_scale=100.0),
        K=16),
}


def n_outlier_channels(cols, frac):
    return int(round(cols * frac))


# ---- host generators (numpy, PCG64) ----------------------------------------

def _to_bf16_bits(x32):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def act_host(rows, cols, seed, dist="normal", outlier_channels=0, outlier_scale=1.0):
    """bf16 activation as uint16 bit patterns, shape [rows, cols]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if dist == "normal":
        x = rng.standard_normal((rows, cols), dtype=np.float32)
    elif dist == "student_t3":
        x = rng.standard_t(3.0, size=(rows, cols)).astype(np.float32)
    else:
        raise ValueError(dist)
    if outlier_channels:
        idx = rng.choice(cols, outlier_channels, replace=False)
        x[:, idx] *= np.float32(outlier_scale)
    return _to_bf16_bits(x)


def grad_host(n, seed, sigma, spike_frac=0.0, spike_scale=1.0):
    """fp32 gradient, shape [n]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    g = rng.standard_normal(n, dtype=np.float32)
    g *= np.float32(sigma)
    if spike_frac > 0.0:
        mask = rng.random(n, dtype=np.float32) < np.float32(spike_frac)
        g[mask] *= np.float32(spike_scale)
    return g


# ---- device generators (torch, seeded generator on the GPU) ----------------

def act_device(rows, cols, seed, dist="normal", outlier_channels=0, outlier_scale=1.0,
               device="cuda"):
    """bf16 activation tensor [rows, cols] generated on the device."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = torch.randn((rows, cols), generator=gen, device=device, dtype=torch.float32)
    if dist == "student_t3":
        chi2 = torch.zeros_like(x)
        for _ in range(3):
            z = torch.randn((rows, cols), generator=gen, device=device, dtype=torch.float32)
            chi2.addcmul_(z, z)
            del z
        x.div_(chi2.div_(3.0).sqrt_())
        del chi2
    elif dist != "normal":
        raise ValueError(dist)
    if outlier_channels:
        idx = torch.randperm(cols, generator=gen, device=device)[:outlier_channels]
        x[:, idx] *= outlier_scale
    return x.to(torch.bfloat16)


def grad_device(n, seed, sigma, spike_frac=0.0, spike_scale=1.0, device="cuda"):
    """fp32 gradient tensor [n] generated on the device."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    g = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    g.mul_(sigma)
    if spike_frac > 0.0:
        mask = torch.rand(n, generator=gen, device=device, dtype=torch.float32) < spike_frac
        g[mask] *= spike_scale
        del mask
    return g
