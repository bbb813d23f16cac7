"""Reduced versions of the five configurations for tests that must finish in seconds on
the CPU, plus a cache so that an archive is generated once per session."""
import functools

from synth import make_config

SMALL = {
    1: {},
    2: dict(layers=6, batch_sizes=[1, 2, 8, 16, 64, 128, 136, 512]),
    3: dict(layers=5, batch_sizes=[1, 4, 16, 24, 256], n_maps=8),
    4: dict(n_words=1 << 20, n_alloc=1 << 16),
    5: dict(layers=6, batch_sizes=[1, 2, 8, 16, 64, 128, 136, 512], n_maps=5),
}


@functools.lru_cache(maxsize=None)
def small(idx):
    return make_config(idx, **SMALL[idx])


@functools.lru_cache(maxsize=2)
def full(idx):
    return make_config(idx)
