"""Seeded synthetic workloads: parameter layouts and input generators.

This module holds NO arithmetic of the method (no accumulation, no selection,
no per-tensor counts): it only produces tensor layouts and random inputs with
the shapes and value distributions of the paper's workloads (Section 5.1 names
ResNet-18/50 on CIFAR-10 and a 5-layer LSTM on AN4; the datasets themselves are
not used, only parameter-tensor shapes).  Both the CPU oracle's tests and the
HIP path's tests/benchmark draw their inputs from here, so that the two
implementations see byte-identical arrays.

All generators use numpy's PCG64 (`default_rng(seed)`), draw in fp32 and run on
the host.
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# layouts
# ----------------------------------------------------------------------------


def offsets_from_sizes(sizes) -> np.ndarray:
    """Element offsets (J+1, uint64) of J tensors packed back to back."""
    off = np.zeros(len(sizes) + 1, dtype=np.uint64)
    off[1:] = np.cumsum(np.asarray(sizes, dtype=np.uint64))
    return off


def resnet50_shapes():
    """Parameter shapes of a ResNet-50 (ImageNet head), in module order.

    Built from the architecture rule: 7x7 stem, bottleneck stages [3, 4, 6, 3]
    with planes 64/128/256/512 and expansion 4, a 1x1 projection in the first
    block of every stage, an affine normalisation (weight, bias) after every
    convolution, and a 1000-way classifier.  53 conv + 106 norm + 2 fc = 161
    tensors, 25,557,032 parameters.
    """
    shapes = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            out = planes * 4
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,)]
            shapes += [(planes, planes, 3, 3), (planes,), (planes,)]
            shapes += [(out, planes, 1, 1), (out,), (out,)]
            if b == 0:
                shapes += [(out, inplanes, 1, 1), (out,), (out,)]
            inplanes = out
    shapes += [(1000, 2048), (1000,)]
    return shapes


def transformer_shapes():
    """12 encoder layers (fused QKV, projection, two MLP matrices) plus a
    30522x768 embedding: 49 tensors, 108,375,552 parameters."""
    shapes = []
    for _ in range(12):
        shapes += [(768, 2304), (768, 768), (768, 3072), (3072, 768)]
    shapes += [(30522, 768)]
    return shapes


def sizes_of(shapes):
    return [int(np.prod(s)) for s in shapes]


def layout_flat(n: int) -> np.ndarray:
    return offsets_from_sizes([n])


def layout_resnet50() -> np.ndarray:
    return offsets_from_sizes(sizes_of(resnet50_shapes()))


def layout_transformer() -> np.ndarray:
    return offsets_from_sizes(sizes_of(transformer_shapes()))


def layout_equal(n: int, J: int) -> np.ndarray:
    assert n % J == 0
    return offsets_from_sizes([n // J] * J)


# ----------------------------------------------------------------------------
# value generators
# ----------------------------------------------------------------------------


def tensor_scales(J: int, seed: int, lo: float = -4.0, hi: float = -1.0) -> np.ndarray:
    """Per-tensor gradient scale, log-uniform in [10^lo, 10^hi]."""
    rng = np.random.default_rng(seed)
    return (10.0 ** rng.uniform(lo, hi, size=J)).astype(np.float32)


def _scale_inplace(x: np.ndarray, offsets: np.ndarray, scales) -> None:
    for j in range(len(offsets) - 1):
        a, b = int(offsets[j]), int(offsets[j + 1])
        x[a:b] *= np.float32(scales[j])


def gaussian(n: int, rng: np.random.Generator) -> np.ndarray:
    return rng.standard_normal(n, dtype=np.float32)


def gaussian_grads(offsets: np.ndarray, scales, rng: np.random.Generator) -> np.ndarray:
    """g_j = scale_j * N(0,1), one flat fp32 array."""
    x = rng.standard_normal(int(offsets[-1]), dtype=np.float32)
    if scales is not None:
        _scale_inplace(x, offsets, scales)
    return x


def tiled_gaussian_grads(offsets: np.ndarray, scales, rng: np.random.Generator,
                         bases: int = 4, shift: int = 1009) -> np.ndarray:
    """Gaussian gradients for very large layouts of equal tensors: `bases` seeded
    N(0,1) blocks of one tensor's size, rotated by `shift * j` and scaled per
    tensor.  Keeps host generation of 1e9 values to seconds."""
    J = len(offsets) - 1
    nj = int(offsets[1] - offsets[0])
    assert all(int(offsets[j + 1] - offsets[j]) == nj for j in range(J))
    blocks = [rng.standard_normal(nj, dtype=np.float32) for _ in range(bases)]
    g = np.empty(J * nj, np.float32)
    for j in range(J):
        s = np.float32(1.0 if scales is None else scales[j])
        np.multiply(np.roll(blocks[j % bases], shift * j), s, out=g[j * nj:(j + 1) * nj])
    return g


def student_t_grads(offsets: np.ndarray, scales, rng: np.random.Generator,
                    nu: float = 3.0) -> np.ndarray:
    """Heavy-tailed gradients: scale_j * t_nu."""
    n = int(offsets[-1])
    x = np.empty(n, dtype=np.float32)
    step = 1 << 24
    for a in range(0, n, step):
        b = min(n, a + step)
        x[a:b] = rng.standard_t(nu, size=b - a).astype(np.float32)
    if scales is not None:
        _scale_inplace(x, offsets, scales)
    return x


def zero_rows(x: np.ndarray, start: int, rows: int, cols: int, keep_frac: float,
              rng: np.random.Generator) -> None:
    """Make a (rows x cols) block of x row-sparse: only a seeded `keep_frac`
    of the rows stay nonzero, the rest become exact +0."""
    keep = rng.random(rows) < keep_frac
    block = x[start:start + rows * cols].reshape(rows, cols)
    block[~keep, :] = 0.0


def integer_grads(n: int, rng: np.random.Generator, lo: int = -8, hi: int = 8) -> np.ndarray:
    """Small integers as fp32, for tests whose arithmetic must be exact."""
    return rng.integers(lo, hi + 1, size=n).astype(np.float32)


def sparse_payload(offsets: np.ndarray, counts, scales, rng: np.random.Generator):
    """A message shaped like one worker's upload: for tensor j, `counts[j]`
    distinct ascending flat indices inside the tensor with values
    scale_j * N(0,1).  `counts` is supplied by the caller."""
    idx_parts, val_parts = [], []
    for j in range(len(offsets) - 1):
        a, b = int(offsets[j]), int(offsets[j + 1])
        c = int(counts[j])
        if c == 0:
            continue
        if c * 8 < (b - a):
            # rejection sampling of distinct positions for sparse picks
            pick = np.unique(rng.integers(a, b, size=int(c * 1.2) + 16))
            while pick.size < c:
                more = rng.integers(a, b, size=c)
                pick = np.unique(np.concatenate([pick, more]))
            if pick.size > c:
                pick = np.sort(rng.choice(pick, size=c, replace=False))
        else:
            pick = np.sort(rng.choice(b - a, size=c, replace=False) + a)
        v = rng.standard_normal(c, dtype=np.float32)
        if scales is not None:
            v *= np.float32(scales[j])
        idx_parts.append(pick.astype(np.uint32))
        val_parts.append(v)
    if not idx_parts:
        return np.zeros(0, np.uint32), np.zeros(0, np.float32)
    return np.concatenate(idx_parts), np.concatenate(val_parts)


def event_schedule(W: int, events: int, seed: int) -> np.ndarray:
    """Arrival order of asynchronous workers: one worker id per event."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, W, size=events).astype(np.uint32)
