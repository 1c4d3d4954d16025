"""Places a batch's per-sequence K and V tensors in device memory and builds the pointer arrays
xattn_decode takes.  Harness plumbing: no arithmetic of the attention path lives here.

Two placements:
  * xtensor=True   each tensor gets its own reserved virtual range (max_seq_len tokens) whose used
                   prefix is backed by 2 MiB physical chunks mapped in a seeded random order
                   (xtensor_map); the data is copied in with xtensor_upload.
  * xtensor=False  each tensor is an ordinary torch allocation.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np
import torch

from . import binding


class KVStore:
    def __init__(self, ks: Sequence[np.ndarray], vs: Sequence[np.ndarray], device: int = 0,
                 xtensor: bool = False, seed: int = 0, max_seq_len: int = 65536):
        assert len(ks) == len(vs)
        self.device = device
        self.xtensor = xtensor
        self._handles: List[int] = []
        self._keep: List[torch.Tensor] = []
        self.n_chunks = 0
        k_addr, v_addr = [], []
        try:
            for b, (k, v) in enumerate(zip(ks, vs)):
                for which, (arr, addrs) in enumerate(((k, k_addr), (v, v_addr))):
                    arr = np.ascontiguousarray(arr, dtype=np.uint16)
                    if xtensor:
                        row_bytes = int(np.prod(arr.shape[1:])) * 2
                        reserve = max(max_seq_len, arr.shape[0]) * row_bytes
                        base, handle = binding.xtensor_map(reserve, arr.nbytes, seed * 1000003 + 2 * b + which,
                                                           device)
                        self._handles.append(handle)
                        self.n_chunks += -(-arr.nbytes // binding.XTENSOR_CHUNK_BYTES)
                        binding.xtensor_upload(base, arr)
                        addrs.append(base)
                    else:
                        t = torch.from_numpy(arr.view(np.int16)).to("cuda:%d" % device)
                        self._keep.append(t)
                        addrs.append(t.data_ptr())
            dev = "cuda:%d" % device
            self.k_ptrs = torch.tensor(k_addr, dtype=torch.int64).to(dev)
            self.v_ptrs = torch.tensor(v_addr, dtype=torch.int64).to(dev)
            self.k_addr, self.v_addr = k_addr, v_addr
        except Exception:
            self.close()
            raise

    def close(self) -> None:
        torch.cuda.synchronize(self.device)
        for h in self._handles:
            binding.xtensor_unmap(h)
        self._handles = []
        self._keep = []

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False
