"""Helpers for the GPU parity tests: numpy <-> device shard lists.  bf16 travels as uint16 bit patterns."""
import numpy as np
import torch

from oracle import tiling as tl
from synthetic import bf16_bits_to_f64, to_bf16_bits

DEV = "cuda:0"


def np_to_dev(a, bf16=False):
    a = np.ascontiguousarray(a)
    if bf16:
        assert a.dtype == np.uint16
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def dev_to_np(t):
    if t.dtype == torch.bfloat16:
        return t.cpu().view(torch.int16).numpy().view(np.uint16)
    return t.cpu().numpy()


def shards_to_dev(T, t, bf16=False):
    """tile a full array on the host (oracle geometry) and upload each shard"""
    return [np_to_dev(s, bf16) for s in tl.tile(T, t)]


def alloc_shards(rows, cols, t, dtype, fill=None):
    sr, sc = tl.shard_shape(rows, cols, t)
    out = []
    for _ in range(1 << len(t)):
        x = torch.empty((sr, sc), dtype=dtype, device=DEV)
        if fill is not None:
            x.fill_(fill)
        out.append(x)
    return out


def shards_to_np(shards):
    return [dev_to_np(s) for s in shards]


def as_f64(a, bf16):
    return bf16_bits_to_f64(a) if bf16 else a.astype(np.float64)


def gather_full(shards, t, rows, cols):
    """device shards -> full host array (raw dtype); checks replicas are identical"""
    return tl.untile(shards_to_np(shards), t, rows, cols)
