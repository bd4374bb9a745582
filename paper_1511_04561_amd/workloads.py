"""Seeded synthetic inputs for the dq8 codec: shapes and value distributions only.

This module holds none of the codec's arithmetic.  It is the one piece shared by
the tests of the CPU oracle and the tests / benchmark of the HIP library, so that
both sides see the same bytes.

The paper (arXiv 1511.04561, Sec. 3.4) measured on gradients and activations of
MNIST, CIFAR10 and ImageNet networks; those data sets and trained networks are not
available here, so tensors with the same layer shapes and plausible value
distributions stand in for them:

  C1  gradients of the 784-1024-1024-10 MLP of Sec. 3.4, normal with std 1e-3
  C2  gradients of a small convnet, Laplace(0, 5e-4) with 1 % outliers at 50x
  C3  gradients of an AlexNet-shaped net (conv shapes of the appendix's layer
      table, fully connected 9216-4096-4096-1000), 1e-3 * Student-t(3),
      concatenated into one flat bucket of 61 100 840 values
  C4  activations after a rectifier: 128 x 4096 and 1024 x 4096, half exact zeros,
      the rest Exp(1)
  C5  K = 8 independent draws (workers) of the C3 bucket

Every tensor is drawn on the host with numpy's PCG64 generator seeded by
``BASE_SEED + 10000 * config + 100 * worker + tensor_index``, in float64, and cast
to float32.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 151104561

C1_SHAPES = [("W1", (784, 1024)), ("b1", (1024,)), ("W2", (1024, 1024)), ("b2", (1024,)),
             ("W3", (1024, 10)), ("b3", (10,))]
C2_SHAPES = [("conv1.w", (64, 3, 5, 5)), ("conv1.b", (64,)), ("conv2.w", (64, 64, 5, 5)), ("conv2.b", (64,)),
             ("fc1.w", (4096, 384)), ("fc1.b", (384,)), ("fc2.w", (384, 192)), ("fc2.b", (192,)),
             ("fc3.w", (192, 10)), ("fc3.b", (10,))]
C3_SHAPES = [("conv1.w", (64, 3, 11, 11)), ("conv1.b", (64,)), ("conv2.w", (192, 64, 5, 5)), ("conv2.b", (192,)),
             ("conv3.w", (384, 192, 3, 3)), ("conv3.b", (384,)), ("conv4.w", (256, 384, 3, 3)), ("conv4.b", (256,)),
             ("conv5.w", (256, 256, 3, 3)), ("conv5.b", (256,)),
             ("fc6.w", (9216, 4096)), ("fc6.b", (4096,)), ("fc7.w", (4096, 4096)), ("fc7.b", (4096,)),
             ("fc8.w", (4096, 1000)), ("fc8.b", (1000,))]
C4_SHAPES = [("act128", (128, 4096)), ("act1024", (1024, 4096))]

SHAPES = {1: C1_SHAPES, 2: C2_SHAPES, 3: C3_SHAPES, 4: C4_SHAPES, 5: C3_SHAPES}
C3_BLOCK = 4096
C3_NUMEL = 61100840
C5_WORKERS = 8


def numel(shape):
    n = 1
    for d in shape:
        n *= int(d)
    return n


def config_numel(config):
    return sum(numel(s) for _, s in SHAPES[config])


def seed_for(config, tensor_index, worker=0):
    return BASE_SEED + 10000 * config + 100 * worker + tensor_index


def _draw(config, rng, n):
    if config == 1:
        return rng.normal(0.0, 1e-3, n)
    if config == 2:
        v = rng.laplace(0.0, 5e-4, n)
        outlier = rng.random(n) < 0.01
        return np.where(outlier, v * 50.0, v)
    if config in (3, 5):
        return 1e-3 * rng.standard_t(3, n)
    if config == 4:
        v = rng.exponential(1.0, n)
        keep = rng.random(n) < 0.5
        return v * keep
    raise ValueError("unknown config %r" % (config,))


def tensor(config, tensor_index, worker=0, limit=None):
    """Flat float32 tensor ``tensor_index`` of ``config``.  ``limit`` keeps only a prefix."""
    n = numel(SHAPES[config][tensor_index][1])
    rng = np.random.Generator(np.random.PCG64(seed_for(config, tensor_index, worker)))
    v = _draw(config, rng, n).astype(np.float32)
    return v if limit is None else v[:limit]


def tensors(config, worker=0):
    """List of (name, flat float32 array) for every tensor of the config."""
    return [(name, tensor(config, t, worker)) for t, (name, _) in enumerate(SHAPES[config])]


def bucket(config=3, worker=0, threads=8):
    """All tensors of the config concatenated in order into one flat float32 array."""
    idx = range(len(SHAPES[config]))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        parts = list(ex.map(lambda t: tensor(config, t, worker), idx))
    return np.concatenate(parts)


def edge_case_block(kind_of_case, n, seed=0):
    """Small adversarial inputs appended to parity runs (not timed)."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 999000 + seed))
    if kind_of_case == "zeros":
        return np.zeros(n, dtype=np.float32)
    if kind_of_case == "neg_zeros":
        return np.full(n, -0.0, dtype=np.float32)
    if kind_of_case == "denormal_absmax":
        v = rng.integers(-(1 << 20), 1 << 20, n).astype(np.float64) * 2.0 ** -149
        return v.astype(np.float32)
    if kind_of_case == "single_nonzero":
        v = np.zeros(n, dtype=np.float32)
        v[int(rng.integers(0, n))] = np.float32(-3.25e-2)
        return v
    if kind_of_case == "huge":
        return (rng.standard_normal(n) * 1e37).astype(np.float32)
    if kind_of_case == "tiny":
        return (rng.standard_normal(n) * 1e-37).astype(np.float32)
    if kind_of_case == "wide":
        return (rng.standard_normal(n) * np.exp(rng.uniform(-20.0, 0.0, n))).astype(np.float32)
    raise ValueError(kind_of_case)
