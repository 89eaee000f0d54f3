"""CPU oracle for bucketed gradient synchronization.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
HIP path is checked against.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product never does, and this
file imports nothing from the product.

What is computed (paper: "PyTorch Distributed: Experiences on Accelerating
Data Parallel Training", arXiv 2006.15704):

  * Section 3.2.3 / Algorithm 1, constructor: parameters are allocated to
    flat buckets in the reverse order of net.parameters() under a bucket
    size cap c.
  * Algorithm 1, autograd_hook: the gradient of parameter i is copied into
    view = b_i.narrow(offset, size) of its bucket; a bucket whose gradients
    are all ready is marked ready; ready buckets are launched in order.
  * Section 4.2, "Autograd Hook": each bucket keeps a count of pending
    gradients, every hook decrements it, the bucket is ready at zero.
  * Section 2.3 / 3.2.1: AllReduce sums equally sized tensors over all
    participants; DDP turns the sum into the average and writes it back to
    the gradient tensors (the finalizing step described after Algorithm 1).
  * Section 3.2.3, second caveat: parameters that take no part in an
    iteration must not keep their bucket from becoming ready.  Here they
    contribute zeros and receive zeros; with per-replica participation
    (`synchronize_local`) a replica that did not use a parameter contributes
    zeros, and Section 4.2's global bitmap (an OR over the ranks) decides
    whether a parameter's gradients are written at all.
  * Section 3.2.4: under no_sync, gradients of several backward passes
    accumulate into the same tensor and are synchronized once afterwards.
  * Section 6.2.1 (gradient order prediction): the backward order seen by
    the hooks is traced and the parameter-to-bucket mapping is rebuilt to
    follow it (`traced_visit_order`, `assign_buckets_in_order`).

  * Section 6.2.3 (gradient compression): gradients need not travel in the
    parameter's own type.  `compress` is what a rank would send (its fp32
    gradient rounded once to a 16-bit format), `reduce_average_transport` /
    `synchronize_transport` sum the R 16-bit copies in binary32, divide by R
    and deliver the average in the parameter's type (fp32) -- the final
    rounding to 16 bits of the all-16-bit path does not happen.

The method is an exact reorganisation of the plain definition

    out_p[j] = (1/R) * sum_{r=0}^{R-1} g_{r,p}[j]

so `mean_definition_f64` writes that definition out in float64, and the
step-by-step functions (assign, pack, reduce, unpack) follow the paper's
steps so that bucket indices and offsets can be compared bit for bit.
`reduce_average` fixes what the definition leaves open: the sum runs over
r = 0, 1, ..., R-1 in IEEE binary32 (round to nearest even), starts from
the r = 0 value, is divided by float32(R), and is rounded once to the
storage format.

Pins (tests/test_oracle_*.py): the hand-derived Tiny assignment, maximal
greedy-partition brute force, unique-tag round trips, integer-valued inputs
against exact integer arithmetic, the float64 definition within the textbook
summation bound, exhaustive 16-bit conversion checks against library
conversions, the tiny linear-regression mean-gradient identity, the no_sync
identity and hand-worked launch schedules; for the traced-order mapping the
reduction to the pinned default assignment, a hand-worked example, partition
invariants, the earliest-possible-launch property and a brute-force search
over small cases; for the lower-precision transport a hand-worked example, the
identity "its result rounded to the transport format equals the pinned
all-16-bit result", integer inputs against exact arithmetic and the float64
bound.

Not pinned by anything in the paper: absolute timings and the best bucket
size (the paper's curves are figures that are not available) -- "parity
unpinned" for those; they are measured, not checked.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

DT_FP32, DT_FP16, DT_BF16 = 0, 1, 2
ESIZE = {DT_FP32: 4, DT_FP16: 2, DT_BF16: 2}
STORAGE = {DT_FP32: np.float32, DT_FP16: np.float16, DT_BF16: np.uint16}
CAP_WHOLE_MODEL = (1 << 64) - 1


# --------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------
def to_f32(x: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of a storage array to binary32."""
    if dtype == DT_FP32:
        return np.asarray(x, dtype=np.float32)
    if dtype == DT_FP16:
        return np.asarray(x, dtype=np.float16).astype(np.float32)
    if dtype == DT_BF16:
        bits = np.asarray(x, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32)
    raise ValueError(f"unknown dtype code {dtype}")


def from_f32(y: np.ndarray, dtype: int) -> np.ndarray:
    """Round binary32 to the storage format, to nearest, ties to even.
    bf16 is the upper half of binary32: add 0x7FFF plus the lowest kept bit,
    then drop the lower 16 bits; NaN stays NaN (quiet bit set)."""
    y = np.asarray(y, dtype=np.float32)
    if dtype == DT_FP32:
        return y
    if dtype == DT_FP16:
        with np.errstate(over="ignore"):
            return y.astype(np.float16)
    if dtype == DT_BF16:
        u = y.view(np.uint32).astype(np.uint64)
        lsb = (u >> np.uint64(16)) & np.uint64(1)
        rounded = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
        nan = np.isnan(y)
        quiet = ((u >> np.uint64(16)) | np.uint64(0x0040)).astype(np.uint16)
        return np.where(nan, quiet, rounded).astype(np.uint16)
    raise ValueError(f"unknown dtype code {dtype}")


# --------------------------------------------------------------------------
# bucket assignment  (Algorithm 1, constructor; Section 4.2)
# --------------------------------------------------------------------------
@dataclass
class Bucket:
    params: List[int] = field(default_factory=list)  # in fill order
    elems: int = 0
    dtype: int = DT_FP32

    @property
    def nbytes(self) -> int:
        return self.elems * ESIZE[self.dtype]


@dataclass
class Assignment:
    bucket_of: np.ndarray   # int32 [n]
    offset_of: np.ndarray   # int64 [n], in elements from the bucket start
    buckets: List[Bucket]
    numel: np.ndarray       # int64 [n]
    dtype: np.ndarray       # int32 [n]


def assign_buckets(numel: Sequence[int], dtype: Sequence[int],
                   cap_bytes: int) -> Assignment:
    """Visit parameters n-1, n-2, ..., 0.  A parameter joins the open bucket
    unless the bucket is non-empty and would then exceed cap_bytes, or holds
    another element type; in that case the open bucket is closed first.  A
    total equal to the cap fits.  Buckets are numbered in the order they are
    opened, so bucket 0 holds the parameters registered last.  Offsets are
    dense (no padding) and counted in elements."""
    n = len(numel)
    if n != len(dtype):
        raise ValueError("numel and dtype differ in length")
    bucket_of = np.full(n, -1, dtype=np.int32)
    offset_of = np.zeros(n, dtype=np.int64)
    buckets: List[Bucket] = []
    cur: Optional[Bucket] = None
    for i in range(n - 1, -1, -1):
        size = int(numel[i]) * ESIZE[int(dtype[i])]
        if cur is not None and cur.params and (
                cur.nbytes + size > cap_bytes or cur.dtype != int(dtype[i])):
            cur = None
        if cur is None:
            cur = Bucket(dtype=int(dtype[i]))
            buckets.append(cur)
        bucket_of[i] = len(buckets) - 1
        offset_of[i] = cur.elems
        cur.params.append(i)
        cur.elems += int(numel[i])
    return Assignment(bucket_of, offset_of, buckets,
                      np.asarray(numel, dtype=np.int64),
                      np.asarray(dtype, dtype=np.int32))


# --------------------------------------------------------------------------
# bucket assignment from a traced backward order  (Section 6.2.1)
# --------------------------------------------------------------------------
def traced_visit_order(ready_sequence: Sequence[int], n: int) -> List[int]:
    """The order in which a rebuilt mapping visits the parameters: first the
    parameters of the traced iteration in the order their gradients became
    ready, then the ones the trace never saw, in reverse registration order
    (the default guess of Algorithm 1 for everything without evidence)."""
    order: List[int] = []
    seen = set()
    for p in ready_sequence:
        p = int(p)
        if p < 0 or p >= n:
            raise ValueError(f"parameter id {p} out of range")
        if p in seen:
            raise ValueError(f"parameter {p} appears twice in the trace")
        seen.add(p)
        order.append(p)
    for i in range(n - 1, -1, -1):
        if i not in seen:
            order.append(i)
    return order


def assign_buckets_in_order(numel: Sequence[int], dtype: Sequence[int], cap_bytes: int,
                            visit_order: Sequence[int]) -> Assignment:
    """Section 6.2.1: the parameter-to-bucket mapping is updated to follow a
    traced backward order.  The allocation rule is Algorithm 1's, only the
    visiting order changes from n-1, ..., 0 to `visit_order` (a permutation
    of the parameter indices): the open bucket is closed before a parameter
    that would push it past cap_bytes or that has another element type; a
    total equal to the cap fits; buckets are numbered as they are opened;
    offsets are dense and counted in elements."""
    n = len(numel)
    if n != len(dtype):
        raise ValueError("numel and dtype differ in length")
    if sorted(int(i) for i in visit_order) != list(range(n)):
        raise ValueError("visit_order is not a permutation of the parameters")
    bucket_of = np.full(n, -1, dtype=np.int32)
    offset_of = np.zeros(n, dtype=np.int64)
    buckets: List[Bucket] = []
    for i in (int(v) for v in visit_order):
        size = int(numel[i]) * ESIZE[int(dtype[i])]
        start_new = (not buckets
                     or buckets[-1].dtype != int(dtype[i])
                     or buckets[-1].nbytes + size > cap_bytes)
        if start_new:
            buckets.append(Bucket(dtype=int(dtype[i])))
        bk = buckets[-1]
        bucket_of[i] = len(buckets) - 1
        offset_of[i] = bk.elems
        bk.params.append(i)
        bk.elems += int(numel[i])
    return Assignment(bucket_of, offset_of, buckets,
                      np.asarray(numel, dtype=np.int64),
                      np.asarray(dtype, dtype=np.int32))


# --------------------------------------------------------------------------
# pack / reduce / unpack
# --------------------------------------------------------------------------
def pack_bucket(asg: Assignment, b: int, grads: Sequence[np.ndarray],
                unused: Sequence[int] = ()) -> np.ndarray:
    """flat[offset_of[i] + j] = grads[i][j] for every parameter i of bucket
    b (Algorithm 1, autograd_hook: view = b_i.narrow(offset, size);
    view.copy_(grad)).  Parameters listed in `unused` are not read and
    their slots hold zeros."""
    bk = asg.buckets[b]
    flat = np.zeros(bk.elems, dtype=STORAGE[bk.dtype])
    skip = set(int(i) for i in unused)
    for i in bk.params:
        if i in skip:
            continue
        off = int(asg.offset_of[i])
        g = np.asarray(grads[i]).reshape(-1)
        if g.size != int(asg.numel[i]) or g.dtype != STORAGE[bk.dtype]:
            raise ValueError(f"gradient {i} has the wrong size or type")
        flat[off:off + g.size] = g
    return flat


def reduce_average(flats: Sequence[np.ndarray], dtype: int) -> np.ndarray:
    """Elementwise over the R replica copies of one bucket:
    s = x_0; s = s + x_r for r = 1..R-1 (binary32); y = s / float32(R);
    result = y rounded to the storage format."""
    R = len(flats)
    if R < 1:
        raise ValueError("need at least one replica")
    with np.errstate(over="ignore", invalid="ignore"):
        s = to_f32(flats[0], dtype).copy()
        for r in range(1, R):
            s = s + to_f32(flats[r], dtype)
        y = s / np.float32(R)
    return from_f32(y.astype(np.float32), dtype)


def unpack_bucket(asg: Assignment, b: int, avg: np.ndarray,
                  outs: List[Optional[np.ndarray]]) -> None:
    """outs[i][j] = avg[offset_of[i] + j]: the write-back of the averaged
    bucket into the per-parameter gradient tensors (finalizing step)."""
    bk = asg.buckets[b]
    for i in bk.params:
        off = int(asg.offset_of[i])
        outs[i] = np.array(avg[off:off + int(asg.numel[i])], copy=True)


# --------------------------------------------------------------------------
# no_sync accumulation  (Section 3.2.4)
# --------------------------------------------------------------------------
def accumulate(acc: List[np.ndarray], micro: Sequence[Optional[np.ndarray]],
               dtype: Sequence[int]) -> None:
    """acc[i] <- round(acc[i] + micro[i]) for every parameter that produced
    a gradient in this micro-step (micro[i] is not None).  The sum is formed
    in binary32 and stored in the gradient's own format, because a gradient
    tensor has its parameter's type."""
    for i, m in enumerate(micro):
        if m is None:
            continue
        d = int(dtype[i])
        with np.errstate(over="ignore", invalid="ignore"):
            acc[i] = from_f32(to_f32(acc[i], d) + to_f32(m, d), d)


# --------------------------------------------------------------------------
# ready marks and in-order launch  (Algorithm 1 hook; Sections 3.2.3, 4.2)
# --------------------------------------------------------------------------
def launch_schedule(asg: Assignment,
                    ready_sequence: Sequence[int]) -> List[Tuple[int, int]]:
    """Replay a sequence of ready marks.  Returns [(bucket, call)] in launch
    order, where `call` is the position in ready_sequence of the mark that
    made the launch possible, or len(ready_sequence) for buckets that only
    the finalizing step launches (they still hold parameters that were never
    marked).  A bucket is launched when its pending count is zero and every
    lower-numbered bucket has been launched."""
    nb = len(asg.buckets)
    pending = [len(bk.params) for bk in asg.buckets]
    seen = set()
    log: List[Tuple[int, int]] = []
    nxt = 0
    for call, p in enumerate(ready_sequence):
        p = int(p)
        if p < 0 or p >= len(asg.bucket_of):
            raise ValueError(f"parameter id {p} out of range")
        if p in seen:
            raise ValueError(f"parameter {p} marked ready twice")
        seen.add(p)
        pending[int(asg.bucket_of[p])] -= 1
        while nxt < nb and pending[nxt] == 0:
            log.append((nxt, call))
            nxt += 1
    while nxt < nb:
        log.append((nxt, len(ready_sequence)))
        nxt += 1
    return log


# --------------------------------------------------------------------------
# the whole path
# --------------------------------------------------------------------------
def synchronize(numel: Sequence[int], dtype: Sequence[int], cap_bytes: int,
                replica_grads: Sequence[Sequence[np.ndarray]],
                ready_sequence: Optional[Sequence[int]] = None,
                visit_order: Optional[Sequence[int]] = None):
    """One synchronization: assign, then per bucket in launch order pack the
    R replica copies, reduce and average, and unpack.  `replica_grads[r][i]`
    is replica r's gradient of parameter i.  Parameters missing from
    `ready_sequence` (default: all are marked, in reverse registration
    order) are reduced as zeros and are not read.  With `visit_order` the
    buckets are the ones rebuilt from a traced order (Section 6.2.1).
    Returns (outs, assignment, launch_log)."""
    n = len(numel)
    R = len(replica_grads)
    asg = (assign_buckets(numel, dtype, cap_bytes) if visit_order is None
           else assign_buckets_in_order(numel, dtype, cap_bytes, visit_order))
    if ready_sequence is None:
        ready_sequence = list(range(n - 1, -1, -1))
    marked = set(int(p) for p in ready_sequence)
    unused = [i for i in range(n) if i not in marked]
    log = launch_schedule(asg, ready_sequence)
    outs: List[Optional[np.ndarray]] = [None] * n
    for b, _ in log:
        flats = [pack_bucket(asg, b, replica_grads[r], unused) for r in range(R)]
        avg = reduce_average(flats, asg.buckets[b].dtype)
        unpack_bucket(asg, b, avg, outs)
    return outs, asg, log


# --------------------------------------------------------------------------
# lower-precision transport  (Section 6.2.3)
# --------------------------------------------------------------------------
def compress(grad_f32: np.ndarray, transport: int) -> np.ndarray:
    """What a rank sends for a binary32 gradient: every element rounded once,
    to nearest even, to the 16-bit transport format."""
    if transport not in (DT_FP16, DT_BF16):
        raise ValueError("the transport format is fp16 or bf16")
    return from_f32(np.ascontiguousarray(grad_f32, dtype=np.float32), transport)


def reduce_average_transport(flats: Sequence[np.ndarray], transport: int,
                             out_dtype: int = DT_FP32) -> np.ndarray:
    """Elementwise over the R transported copies of one bucket:
    s = float(x_0); s = s + float(x_r) for r = 1..R-1 (binary32);
    y = s / float32(R); the result is y in the parameter's format (for
    binary32 parameters: y itself, no second rounding)."""
    R = len(flats)
    if R < 1:
        raise ValueError("need at least one replica")
    with np.errstate(over="ignore", invalid="ignore"):
        s = to_f32(flats[0], transport).copy()
        for r in range(1, R):
            s = s + to_f32(flats[r], transport)
        y = s / np.float32(R)
    return from_f32(y.astype(np.float32), out_dtype)


def synchronize_transport(numel: Sequence[int], transport: Sequence[int], cap_bytes: int,
                          replica_grads: Sequence[Sequence[np.ndarray]],
                          ready_sequence: Optional[Sequence[int]] = None,
                          out_dtype: int = DT_FP32):
    """One synchronization whose replica gradients are held in a 16-bit
    transport format (`transport[i]`, `replica_grads[r][i]` in that format)
    while the averages are delivered in `out_dtype`.  A bucket is what is
    communicated, so buckets are filled and capped by transport bytes; pack,
    launch order and the handling of parameters that were never marked are
    those of `synchronize`.  Returns (outs, assignment, launch_log)."""
    n = len(numel)
    R = len(replica_grads)
    asg = assign_buckets(numel, transport, cap_bytes)
    if ready_sequence is None:
        ready_sequence = list(range(n - 1, -1, -1))
    marked = set(int(p) for p in ready_sequence)
    unused = [i for i in range(n) if i not in marked]
    log = launch_schedule(asg, ready_sequence)
    outs: List[Optional[np.ndarray]] = [None] * n
    for b, _ in log:
        bk = asg.buckets[b]
        flats = [pack_bucket(asg, b, replica_grads[r], unused) for r in range(R)]
        avg = reduce_average_transport(flats, bk.dtype, out_dtype)
        for i in bk.params:                       # the write-back of unpack_bucket, in the output type
            off = int(asg.offset_of[i])
            outs[i] = np.array(avg[off:off + int(asg.numel[i])], copy=True)
    return outs, asg, log


# --------------------------------------------------------------------------
# per-replica participation and the global bitmap  (Sections 3.2.3, 4.2)
# --------------------------------------------------------------------------
def global_used_bitmap(local_used: np.ndarray) -> np.ndarray:
    """local_used[r][i] = 1 if replica r's backward pass produced a gradient
    for parameter i.  The extra AllReduce on the bitmap tells every rank which
    parameters were used by at least one rank: an OR over the replicas."""
    local_used = np.asarray(local_used, dtype=np.uint8)
    out = np.zeros(local_used.shape[1], dtype=np.uint8)
    for r in range(local_used.shape[0]):
        out = out | (local_used[r] != 0).astype(np.uint8)
    return out


def synchronize_local(numel: Sequence[int], dtype: Sequence[int], cap_bytes: int,
                      replica_grads: Sequence[Sequence[np.ndarray]],
                      marks: Sequence[Tuple[int, Sequence[int]]],
                      find_unused: bool = True,
                      prior_used: Optional[np.ndarray] = None,
                      visit_order: Optional[Sequence[int]] = None):
    """One synchronization in which every replica has its own set of used
    parameters.  `marks` is the sequence of ready marks, each (parameter,
    used[R]); `prior_used[r][i]` (optional) carries participation recorded by
    earlier no_sync iterations, which the paper lets accumulate in the bitmap
    until the next communication.  A replica that did not use a parameter
    contributes zeros for it and its tensor is not read; the sum is still
    divided by R (DDP always averages over all processes).  A parameter that
    no replica used is globally unused: with find_unused its gradients stay as
    they are, otherwise they become zeros.
    Returns (outs[R][n] -- every replica's view of its gradient tensors after
    the synchronization --, assignment, launch_log, global_used)."""
    n, R = len(numel), len(replica_grads)
    asg = (assign_buckets(numel, dtype, cap_bytes) if visit_order is None
           else assign_buckets_in_order(numel, dtype, cap_bytes, visit_order))
    local = np.zeros((R, n), dtype=np.uint8) if prior_used is None else (np.asarray(prior_used) != 0).astype(np.uint8)
    order = []
    for p, used in marks:
        order.append(int(p))
        for r in range(R):
            if used[r]:
                local[r, int(p)] = 1
    log = launch_schedule(asg, order)
    glob = global_used_bitmap(local)
    outs = [[np.array(replica_grads[r][i], copy=True) for i in range(n)] for r in range(R)]
    for b, _ in log:
        flats = [pack_bucket(asg, b, replica_grads[r], [i for i in asg.buckets[b].params if not local[r, i]])
                 for r in range(R)]
        avg = reduce_average(flats, asg.buckets[b].dtype)
        res: List[Optional[np.ndarray]] = [None] * n
        unpack_bucket(asg, b, avg, res)
        for i in asg.buckets[b].params:
            if glob[i] or not find_unused:
                for r in range(R):
                    outs[r][i] = res[i].copy()
    return outs, asg, log, glob


def mean_definition_f64(replica_grads: Sequence[Sequence[np.ndarray]],
                        dtype: Sequence[int]) -> List[np.ndarray]:
    """The plain definition, out_p = (1/R) sum_r g_{r,p}, in float64 and
    without any bucketing."""
    R = len(replica_grads)
    outs = []
    for i in range(len(replica_grads[0])):
        acc = np.zeros(np.asarray(replica_grads[0][i]).size, dtype=np.float64)
        for r in range(R):
            acc += to_f32(replica_grads[r][i], int(dtype[i])).astype(np.float64).reshape(-1)
        outs.append(acc / R)
    return outs
