"""Shared test helpers: numpy uint64 <-> torch int64 on the GPU."""
import numpy as np
import torch

P61 = (1 << 61) - 1


def to_dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return torch.from_numpy(a.view(np.int64)).to("cuda:0")


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy().view(np.uint64)


def field_uniform(shape, seed, edge=True) -> np.ndarray:
    """uniform field elements with a few extreme values planted"""
    rng = np.random.default_rng(seed)
    a = rng.integers(0, P61, size=shape, dtype=np.uint64)
    if edge and a.size >= 8:
        flat = a.reshape(-1)
        flat[0], flat[1], flat[2], flat[3] = 0, P61 - 1, 1, (P61 - 1) // 2
        flat[-1], flat[-2] = P61 - 1, 0
    return a
