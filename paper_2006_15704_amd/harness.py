"""Device-memory and stream plumbing around the C-ABI binding, used by the GPU
tests, the smoke check and the benchmark.  PyTorch is used for exactly two
things here: allocating device memory and creating streams.  Nothing in this
file computes on gradients; every step of the synchronization path runs in the
library's HIP kernels.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B

ESIZE = {B.DDP_FP32: 4, B.DDP_FP16: 2, B.DDP_BF16: 2}
NP_STORAGE = {B.DDP_FP32: np.float32, B.DDP_FP16: np.float16, B.DDP_BF16: np.uint16}


def require_gpu() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
    return torch.device("cuda:0")


class DeviceGrads:
    """R x n gradient tensors in device memory.  Each replica is one byte
    buffer; tensor i of every replica starts at the same offset, aligned to
    `align` bytes plus an optional per-tensor skew (in bytes, a multiple of the
    element size) that tests use to produce tensors that are not 16-byte
    aligned."""

    def __init__(self, numel: Sequence[int], dtype: Sequence[int], R: int,
                 align: int = 256, skew: Optional[Sequence[int]] = None,
                 replica_skew: Optional[Sequence[int]] = None, fill: Optional[int] = None):
        self.device = require_gpu()
        self.numel = [int(x) for x in numel]
        self.dtype = [int(x) for x in dtype]
        self.n, self.R = len(self.numel), int(R)
        self.offsets: List[int] = []
        off = 0
        for i, (ne, dt) in enumerate(zip(self.numel, self.dtype)):
            off = (off + align - 1) // align * align
            if skew is not None:
                assert skew[i] % ESIZE[dt] == 0
                off += int(skew[i])
            self.offsets.append(off)
            off += ne * ESIZE[dt]
        self.slab_bytes = off + 64
        self.replica_skew = [0] * self.R if replica_skew is None else [int(x) for x in replica_skew]
        self.bufs = []
        for r in range(self.R):
            buf = torch.empty(self.slab_bytes + 64, dtype=torch.uint8, device=self.device)
            if fill is not None:
                buf.fill_(fill)
            self.bufs.append(buf)

    def nbytes(self, i: int) -> int:
        return self.numel[i] * ESIZE[self.dtype[i]]

    def view(self, r: int, i: int) -> torch.Tensor:
        o = self.offsets[i] + self.replica_skew[r]
        return self.bufs[r][o:o + self.nbytes(i)]

    def ptr(self, r: int, i: int) -> int:
        return self.bufs[r].data_ptr() + self.offsets[i] + self.replica_skew[r]

    def ptrs(self) -> List[int]:
        return [self.ptr(r, i) for r in range(self.R) for i in range(self.n)]

    def upload(self, r: int, i: int, host: np.ndarray) -> None:
        host = np.ascontiguousarray(host)
        assert host.dtype == NP_STORAGE[self.dtype[i]] and host.size == self.numel[i]
        if host.size:
            self.view(r, i).copy_(torch.from_numpy(host.view(np.uint8).reshape(-1)))

    def upload_replica(self, r: int, host_list: Sequence[np.ndarray]) -> None:
        for i, h in enumerate(host_list):
            self.upload(r, i, h)

    def download(self, r: int, i: int) -> np.ndarray:
        raw = self.view(r, i).cpu().numpy()
        return raw.view(NP_STORAGE[self.dtype[i]]).copy()

    def fill_bytes(self, r: int, i: int, byte: int) -> None:
        if self.nbytes(i):
            self.view(r, i).fill_(byte)


class Session:
    """A context with its two streams.  Thin convenience over the binding."""

    def __init__(self, grads: DeviceGrads, cap_bytes: int, pipeline: int = B.DDP_PIPELINE_STAGED,
                 write_all: bool = False, same_stream: bool = False, streams=None,
                 outputs: Optional[DeviceGrads] = None):
        """outputs: a one-replica binary32 DeviceGrads of the same numel that receives the
        averages of 16-bit gradients (ddp_set_outputs)."""
        self.grads = grads
        self.outputs = outputs
        self.pipeline = pipeline
        self.ctx = None
        # HIP streams that share a hardware queue run one after the other: a reduction stream
        # like that overlaps nothing.  The library probes the pair it is given
        # (DDP_OPT_FLAG_ORDER reads 1 if the streams run concurrently); new streams are tried
        # until a pair passes, the last pair is used as it is.
        for attempt in range(8):
            if streams is not None:      # (reduce, backward) of another session: contexts that share them
                self.reduce_stream, self.backward_stream = streams
            elif attempt == 0 or not same_stream:
                self.reduce_stream = torch.cuda.Stream(device=grads.device)
                self.backward_stream = self.reduce_stream if same_stream else torch.cuda.Stream(device=grads.device)
            torch.cuda.synchronize()
            self.ctx = B.ddp_create(grads.R, 0, self.reduce_stream.cuda_stream,
                                    self.backward_stream.cuda_stream)
            B.ddp_set_option(self.ctx, B.DDP_OPT_PIPELINE, pipeline)
            B.ddp_set_option(self.ctx, B.DDP_OPT_WRITE_ALL, 1 if write_all else 0)
            B.ddp_register_params(self.ctx, grads.numel, grads.dtype, grads.ptrs())
            if outputs is not None:
                B.ddp_set_outputs(self.ctx, [outputs.ptr(0, i) for i in range(outputs.n)])
            self.n_buckets = B.ddp_build_buckets(self.ctx, cap_bytes)
            self.streams_concurrent = bool(B.ddp_get_option(self.ctx, B.DDP_OPT_FLAG_ORDER))
            if (self.streams_concurrent or streams is not None or same_stream
                    or pipeline != B.DDP_PIPELINE_FUSED or attempt == 7):
                break
            B.ddp_destroy(self.ctx)
            self.ctx = None

    def sync(self, ready_order: Optional[Sequence[int]] = None, one_by_one: bool = False) -> None:
        """mark every parameter of ready_order (default: reverse registration
        order), finalize, wait."""
        if ready_order is None:
            ready_order = range(self.grads.n - 1, -1, -1)
        if one_by_one:
            for p in ready_order:
                B.ddp_mark_ready(self.ctx, int(p))
        else:
            B.ddp_mark_ready_many(self.ctx, list(ready_order))
        B.ddp_finalize_backward(self.ctx)
        B.ddp_synchronize(self.ctx)

    def bucket_bytes(self, b: int, r: int) -> np.ndarray:
        """Raw bytes of bucket b's flat buffer of replica r (-1: the average)."""
        elems, _, dt = B.ddp_get_bucket_info(self.ctx, b)
        nbytes = elems * ESIZE[dt]
        ptr = B.ddp_get_bucket_ptr(self.ctx, b, r)
        if nbytes == 0:
            return np.zeros(0, dtype=NP_STORAGE[dt])

        class _Raw:   # lets torch wrap library-owned device memory without copying
            __cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1",
                                        "data": (ptr, False), "version": 2}
        raw = torch.as_tensor(_Raw(), device=self.grads.device)
        return raw.cpu().numpy().view(NP_STORAGE[dt]).copy()

    def close(self) -> None:
        if self.ctx is not None:
            B.ddp_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
