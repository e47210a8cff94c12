"""Small helpers shared by the tests (no method arithmetic)."""
import numpy as np
import torch

from paper_2411_01611_amd import synth


def np_tables(wl, tables):
    """torch CPU tables -> numpy arrays the oracle takes (bf16 as uint16 bit patterns)."""
    if wl.dtype == "f32":
        return [t.numpy() for t in tables]
    return [t.view(torch.int16).numpy().view(np.uint16) for t in tables]


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


def small_workload(name="tiny", **over):
    return synth.workload(name, **over)


def gids_of(wl, indices, offsets):
    """Global row id of every lookup, from the table-major layout (numpy, for test-side brute force)."""
    B, T = wl.batch, wl.num_tables
    rb = wl.row_base
    out = np.empty(indices.shape[0], dtype=np.int64)
    for t in range(T):
        a, b = int(offsets[t * B]), int(offsets[(t + 1) * B])
        out[a:b] = rb[t] + indices[a:b].astype(np.int64)
    return out


def bag_of(offsets, L):
    """Bag id of every lookup position."""
    lens = np.diff(offsets.astype(np.int64))
    return np.repeat(np.arange(lens.shape[0], dtype=np.int64), lens)
