"""Seeded synthetic gradients shaped like the paper's three training workloads.

The paper trains ResNet101 (170 MB), a 2-layer LSTM (252 MB) and VGG16 (528 MB)
on CIFAR10 / PTB / CIFAR100 (Table I).  Those datasets, weights and real
gradients are not available here; the generators below stand in for them with
the same tensor shapes and a stated value distribution.  They are pure input
generators: none of the method's arithmetic (error feedback, selection,
statistics) lives here, so both the GPU path and the CPU oracle may be fed from
this module.

All generators draw from ``numpy.random.Generator(PCG64(seed))`` in float64 and
cast once to float32.
"""
from __future__ import annotations

import numpy as np

_CHUNK = 1 << 24  # elements drawn per call, bounds the float64 temporaries


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _fill(out: np.ndarray, draw) -> None:
    """out[:] = draw(m) cast to float32, in bounded chunks (draw returns float64[m])."""
    n = out.size
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        out[s:s + m] = draw(m).astype(np.float32)


# --------------------------------------------------------------------------
# tensor lists
# --------------------------------------------------------------------------

def resnet101_tensor_sizes() -> list[int]:
    """Parameter tensors of ResNet-101 (ImageNet head) in definition order.

    Stem 7x7x3->64 conv and its two batch-norm vectors; four bottleneck stages of
    3 / 4 / 23 / 3 blocks with widths 64 / 128 / 256 / 512, each block being
    1x1 in->w, 3x3 w->w, 1x1 w->4w convolutions, every convolution followed by
    two batch-norm vectors of its output width; the first block of a stage adds a
    1x1 in->4w projection with its two batch-norm vectors; then the 2048->1000
    classifier weight and bias.  314 tensors, 44,549,160 elements (Table I: 170 MB).
    """
    sizes = [7 * 7 * 3 * 64, 64, 64]
    cin = 64
    for blocks, w in ((3, 64), (4, 128), (23, 256), (3, 512)):
        for b in range(blocks):
            sizes += [cin * w, w, w, 9 * w * w, w, w, w * 4 * w, 4 * w, 4 * w]
            if b == 0:
                sizes += [cin * 4 * w, 4 * w, 4 * w]
            cin = 4 * w
    sizes += [2048 * 1000, 1000]
    return sizes


def vgg16_tensor_sizes() -> list[int]:
    """VGG16 parameter tensors: 13 conv weights+biases, then 3 fully connected layers.

    138,357,544 elements (Table I: 528 MB); the last six tensors (fc weights and
    biases) hold 123,642,856 of them.
    """
    cfg = [64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]
    sizes = []
    cin = 3
    for c in cfg:
        sizes += [9 * cin * c, c]
        cin = c
    sizes += [25088 * 4096, 4096, 4096 * 4096, 4096, 4096 * 1000, 1000]
    return sizes


def lstm_tensor_sizes(vocab: int = 33278, hidden: int = 650) -> list[int]:
    """2-layer LSTM language model: embedding, per layer W_ih, W_hh, b_ih, b_hh, decoder W and b."""
    sizes = [vocab * hidden]
    for _ in range(2):
        sizes += [4 * hidden * hidden, 4 * hidden * hidden, 4 * hidden, 4 * hidden]
    sizes += [vocab * hidden, vocab]
    return sizes


def offsets_of(sizes) -> np.ndarray:
    """int64 offsets [0, s0, s0+s1, ...] of consecutive tensors in the flat gradient."""
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(np.asarray(sizes, dtype=np.int64), out=off[1:])
    return off


# --------------------------------------------------------------------------
# value generators
# --------------------------------------------------------------------------

def normal_gradient(n: int, sigma: float, seed: int) -> np.ndarray:
    """iid Normal(0, sigma) gradient."""
    rng = _rng(seed)
    out = np.empty(n, dtype=np.float32)
    _fill(out, lambda m: rng.standard_normal(m) * sigma)
    return out


def resnet_like_gradient(n: int, seed: int, scale: float = 1e-4,
                         outlier_frac: float = 0.01, outlier_gain: float = 100.0) -> np.ndarray:
    """Laplace(0, scale) values, a seeded `outlier_frac` of positions multiplied by `outlier_gain`."""
    rng = _rng(seed)
    out = np.empty(n, dtype=np.float32)

    def draw(m):
        v = rng.laplace(0.0, scale, m)
        hit = rng.random(m) < outlier_frac
        v[hit] *= outlier_gain
        return v

    _fill(out, draw)
    return out


def vgg_like_gradient(n_conv: int, n_fc: int, seed: int,
                      sigma_conv: float = 1e-3, sigma_fc: float = 1e-5) -> np.ndarray:
    """Convolution part first (Normal(0, sigma_conv)), then the fc part (Normal(0, sigma_fc))."""
    rng = _rng(seed)
    out = np.empty(n_conv + n_fc, dtype=np.float32)
    _fill(out[:n_conv], lambda m: rng.standard_normal(m) * sigma_conv)
    _fill(out[n_conv:], lambda m: rng.standard_normal(m) * sigma_fc)
    return out


def lstm_like_gradient(seed: int, vocab: int = 33278, hidden: int = 650,
                       zero_row_frac: float = 0.95, sigma: float = 1e-4) -> np.ndarray:
    """LSTM LM gradient: whole embedding rows exactly +0.0 for a seeded 95 % of the
    vocabulary (tokens absent from the batch), everything else Normal(0, sigma)."""
    rng = _rng(seed)
    sizes = lstm_tensor_sizes(vocab, hidden)
    out = np.empty(sum(sizes), dtype=np.float32)
    _fill(out, lambda m: rng.standard_normal(m) * sigma)
    n_live = vocab - int(round(vocab * zero_row_frac))
    live = rng.choice(vocab, size=n_live, replace=False)
    dead = np.ones(vocab, dtype=bool)
    dead[live] = False
    emb = out[:vocab * hidden].reshape(vocab, hidden)
    emb[dead, :] = 0.0
    return out


# --------------------------------------------------------------------------
# the five benchmark configurations (full size) and reduced twins for the oracle
# --------------------------------------------------------------------------

VGG16_N_CONV = 14_714_688
VGG16_N_FC = 123_642_856
RESNET101_N = 44_549_160
LSTM_N = 50_065_078


def config1(iteration: int, n: int = 1 << 20) -> np.ndarray:
    """N = 2^20, Normal(0, 1e-3), seed = iteration; residual starts at zero; CF 100."""
    return normal_gradient(n, 1e-3, iteration)


def config2_grad(iteration: int, n: int = RESNET101_N) -> np.ndarray:
    """ResNet101-shaped: Laplace(0, 1e-4), 1 % outliers x100; seed = iteration."""
    return resnet_like_gradient(n, iteration)


def config2_residual0(n: int = RESNET101_N) -> np.ndarray:
    """Initial residual of config 2: Normal(0, 1e-5), seed 1000."""
    return normal_gradient(n, 1e-5, 1000)


def config3_grad(iteration: int, n_conv: int = VGG16_N_CONV, n_fc: int = VGG16_N_FC) -> np.ndarray:
    """VGG16-shaped: conv part Normal(0, 1e-3) then fc part Normal(0, 1e-5); seed = iteration."""
    return vgg_like_gradient(n_conv, n_fc, iteration)


def config4_grad(seed: int = 0, vocab: int = 33278, hidden: int = 650) -> np.ndarray:
    """2-layer LSTM LM gradient with 95 % zero embedding rows."""
    return lstm_like_gradient(seed, vocab, hidden)


def config5_worker_grad(worker: int, n: int = RESNET101_N) -> np.ndarray:
    """Worker w's ResNet101-shaped gradient (seed = worker), split by resnet101_tensor_sizes()."""
    return resnet_like_gradient(n, worker)


def scaled_sizes(sizes, divisor: int, floor: int = 1) -> list[int]:
    """Shrink a tensor list for CPU-sized tests, keeping count, order and small tensors."""
    return [max(floor, s // divisor) if s > 4096 else s for s in sizes]
