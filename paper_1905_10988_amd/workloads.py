"""Seeded synthetic gradients shaped like the paper's workloads.

This module only draws inputs (numpy, fixed seeds).  It holds none of the
compression arithmetic and imports neither the GPU binding nor the CPU oracle,
so both sides can be fed the very same bytes.

The paper measures on gradients of real networks (a 100 MB-per-tensor
aggregation micro-benchmark, ResNet/VGG/AlexNet training).  Those models and
their gradients are not available here; the generators below stand in for them
with the same sizes, per-layer structure and value ranges (exponents of real
gradients stay within about 2^-50 .. 2^10, App. B exponent histograms).
"""
import math

import numpy as np

# Sizes named by the benchmark configurations.
D_SMALL = 1_048_576            # config 1
D_RESNET50 = 25_557_032        # configs 2 and 3 (a ResNet-50-sized parameter count)
D_VGG16 = 138_357_544          # config 4 (a VGG-16-sized parameter count)
NUM_LAYERS = 161
LAYER_MIN, LAYER_MAX = 64, 2_359_296
BUCKET = 8192
NUM_WORKERS = 8


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _log_uniform(rng, lo, hi, size):
    return np.exp(rng.uniform(math.log(lo), math.log(hi), size))


def layer_offsets(d=D_RESNET50, num_layers=NUM_LAYERS, lo=LAYER_MIN, hi=LAYER_MAX, seed=1002):
    """Offsets (num_layers+1, uint64) of contiguous layer tensors whose lengths are
    log-uniform in [lo, hi], rescaled so that they sum to d."""
    assert num_layers * lo <= d
    rng = _rng(seed)
    raw = _log_uniform(rng, lo, hi, num_layers)
    hi_eff = max(hi, -(-d // num_layers))
    lengths = np.clip(np.rint(raw * (d / raw.sum())), lo, hi_eff).astype(np.int64)
    # hand the rounding residual to (or take it from) the largest layers, one pass at a time
    order = np.argsort(-lengths, kind="stable")
    residual = int(d - lengths.sum())
    guard = 0
    while residual != 0:
        for j in order:
            if residual == 0:
                break
            room = (hi_eff - lengths[j]) if residual > 0 else (lengths[j] - lo)
            step = int(np.sign(residual)) * min(abs(residual), int(room))
            lengths[j] += step
            residual -= step
        guard += 1
        assert guard < 64, "could not distribute the residual"
    off = np.zeros(num_layers + 1, np.uint64)
    off[1:] = np.cumsum(lengths).astype(np.uint64)
    assert int(off[-1]) == d
    return off


def config1(d=D_SMALL, seed=0):
    """N(0,1)*1e-3 with 1 % exact +-powers of two and 0.1 % exact zeros (pass-through cases)."""
    rng = _rng(seed)
    x = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    n_pow = max(d // 100, 1)
    n_zero = max(d // 1000, 1)
    pos = rng.permutation(d)[: n_pow + n_zero]
    exps = rng.integers(-30, -5, n_pow)                     # the bulk of the data lies in 2^-30 .. 2^-6
    signs = rng.integers(0, 2, n_pow) * 2.0 - 1.0
    x[pos[:n_pow]] = (signs * np.exp2(exps.astype(np.float64))).astype(np.float32)
    zeros = np.zeros(n_zero, np.float32)
    zeros[rng.integers(0, 2, n_zero) == 1] = -0.0
    x[pos[n_pow:]] = zeros
    return x


def layered_gaussian(worker, offsets, sigma_lo=1e-5, sigma_hi=1e-1, seed=1002):
    """Config 2: worker `worker`'s gradient; layer l is N(0, sigma_l^2), sigma_l log-uniform,
    the same sigma_l for every worker."""
    nl = offsets.size - 1
    sigma = _log_uniform(_rng(seed + 7919), sigma_lo, sigma_hi, nl)
    rng = _rng([seed, 1 + worker])
    d = int(offsets[-1])
    x = rng.standard_normal(d, dtype=np.float32)
    x *= np.repeat(sigma, np.diff(offsets.astype(np.int64))).astype(np.float32)
    return x


def layered_laplace(worker, offsets, b_lo=1e-5, b_hi=1e-2, seed=1003):
    """Config 3: layer l is Laplace(0, b_l), b_l log-uniform."""
    nl = offsets.size - 1
    b = _log_uniform(_rng(seed + 7919), b_lo, b_hi, nl)
    rng = _rng([seed, 1 + worker])
    d = int(offsets[-1])
    x = rng.laplace(0.0, 1.0, d).astype(np.float32)
    x *= np.repeat(b, np.diff(offsets.astype(np.int64))).astype(np.float32)
    return x


def bucketed_gaussian(worker, d=D_VGG16, bucket=BUCKET, scale_lo=1e-6, scale_hi=1e-1, seed=1004):
    """Config 4: N(0,1) times a per-bucket scale, log-uniform, shared by the workers."""
    nb = -(-d // bucket)
    scale = _log_uniform(_rng(seed + 7919), scale_lo, scale_hi, nb).astype(np.float32)
    rng = _rng([seed, 1 + worker])
    x = rng.standard_normal(d, dtype=np.float32)
    x *= np.repeat(scale, bucket)[:d]
    return x


D_BERT_LARGE = 335_000_000     # config 5 (a BERT-large-sized parameter count)


def dense_gaussian(worker, d=D_BERT_LARGE, sigma=1e-2, seed=1005):
    """Config 5: entries i.i.d. N(0, 1e-4) (sigma = 1e-2)."""
    rng = _rng([seed, 1 + worker])
    x = rng.standard_normal(d, dtype=np.float32)
    x *= np.float32(sigma)
    return x


def edge_values():
    """A short vector of binary32 corner cases: signed zeros, subnormals, exact powers of
    two, values next to powers of two, the largest finite value, infinities and a NaN."""
    bits = np.array([
        0x00000000, 0x80000000,             # +-0
        0x00000001, 0x80000001, 0x007FFFFF, 0x00400000,   # subnormals
        0x00800000, 0x80800000,             # smallest normal
        0x3F800000, 0xBF800000, 0x40000000, 0x3F000000,   # +-1, 2, 0.5
        0x3F800001, 0x3FFFFFFF, 0xBFFFFFFF, # just above 1, just below 2
        0x40200000, 0xC0300000, 0x3F400000, # 2.5, -2.75, 0.75
        0x3FAAAAAB,                         # 4/3, the worst case of the variance bound
        0x7F7FFFFF, 0xFF7FFFFF,             # +-largest finite
        0x7F000000,                         # 2^127
        0x7F800000, 0xFF800000, 0x7FC00000, # +-Inf, NaN
    ], dtype=np.uint32)
    return bits.view(np.float32).copy()


# --------------------------------------------------------------------------- device-side variants
# The throughput benchmark times configurations 3 and 4 (up to 4.4 GB of input) on inputs drawn
# directly on the GPU with the same recipes; parity tests use the numpy generators above.
def layered_laplace_device(worker, offsets, b_lo=1e-5, b_hi=1e-2, seed=1003, device="cuda"):
    import torch
    nl = offsets.size - 1
    b = _log_uniform(_rng(seed + 7919), b_lo, b_hi, nl).astype(np.float32)
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + worker)
    d = int(offsets[-1])
    u = torch.rand(d, device=device, generator=g) - 0.5
    x = -torch.sign(u) * torch.log1p(-2 * u.abs())               # inverse CDF of Laplace(0, 1)
    scale = torch.repeat_interleave(torch.from_numpy(b).to(device),
                                    torch.from_numpy(np.diff(offsets.astype(np.int64))).to(device))
    return (x * scale).contiguous()


def bucketed_gaussian_device(worker, d=D_VGG16, bucket=BUCKET, scale_lo=1e-6, scale_hi=1e-1, seed=1004, device="cuda",
                             out=None):
    import torch
    nb = -(-d // bucket)
    scale = _log_uniform(_rng(seed + 7919), scale_lo, scale_hi, nb).astype(np.float32)
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + worker)
    x = torch.empty(d, dtype=torch.float32, device=device) if out is None else out
    x.normal_(generator=g)
    x *= torch.repeat_interleave(torch.from_numpy(scale).to(device), bucket)[:d]
    return x


def dense_gaussian_device(worker, d=D_BERT_LARGE, sigma=1e-2, seed=1005, device="cuda", out=None):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + worker)
    x = torch.empty(d, dtype=torch.float32, device=device) if out is None else out
    x.normal_(0.0, sigma, generator=g)
    return x
