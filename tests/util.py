"""Shared helpers of the tests: cached blobs, oracle models and GPU flows."""
import functools

import numpy as np

from synth import CONFIGS, make_blob, make_images


@functools.lru_cache(maxsize=4)
def blob_of(name, mode="random"):
    return make_blob(CONFIGS[name], mode=mode)


def oracle_model(name, mode="random"):
    import oracle
    return oracle.Model(blob_of(name, mode))


def gpu_flow(name, max_batch, mode="random"):
    import paper_2206_08869_amd as iodf
    return iodf.Flow(blob_of(name, mode), max_batch=max_batch, device=0)


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def images(name, batch=None, kind=None):
    return make_images(CONFIGS[name], batch=batch, kind=kind)
