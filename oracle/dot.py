"""CPU oracle: the contraction each partition must reproduce.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file.
It shares no code with the HIP/C++ library.

What it states:

* Section 3.2: an Einsum / XLA Dot is a generalised matrix multiply whose
  dimensions are batch (in both operands and the output), contracting (in both
  operands, summed away) or non-contracting (in one operand and the output):
      OUT[b.., i.., j..] = sum_{c..} LHS[b.., i.., c..] * RHS[b.., c.., j..]
  The output dimension order is batch, lhs non-contracting, rhs non-contracting
  (the paper leaves the order open; this is the reading taken).
* Section 1 / Section 4: the partitioned program is mathematically equivalent
  to the unpartitioned one.  So what partition p must hold is a *slice* of OUT
  at its shard offset, and for a mesh axis that splits a contracting dimension
  it holds the dot over its slice of that dimension, the partials summing to
  OUT (the AllReduce of Section 4.2).
* Section 4.1: padded positions are replaced by the identity of the reduction
  (0 for a sum) before they can contribute.
* Section 4.2: a ReduceScatter is an AllReduce followed by each partition's
  DynamicSlice of the reduced data.  So a partition whose out sharding splits an
  output dimension over the mesh dimension that carries the sum must hold
  `expected_out_shard(full sum, out mapping)`; no separate function is needed.
* Section 5.1: the feed-forward layer is Relu(x W_in) W_out with an elementwise
  Relu, max(x, 0), applied to the finished (fully summed) first product.

Arithmetic is float64 on the exact input values (bf16 or fp32 widened without
rounding).  No blocking, fusion or reordering beyond the definition: operands
are transposed to [batch, free, contract] / [batch, contract, free], flattened,
and multiplied with numpy's float64 matmul.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

from . import bounds as _bounds


def _free_dims(rank: int, batch: Sequence[int], contract: Sequence[int]):
    return [d for d in range(rank) if d not in batch and d not in contract]


def dot_general(lhs: np.ndarray, rhs: np.ndarray,
                lhs_batch: Sequence[int], rhs_batch: Sequence[int],
                lhs_contract: Sequence[int], rhs_contract: Sequence[int]) -> np.ndarray:
    """Unpartitioned float64 dot_general (Section 3.2); output [batch, lhs free, rhs free]."""
    lhs = np.asarray(lhs, dtype=np.float64)
    rhs = np.asarray(rhs, dtype=np.float64)
    if len(lhs_batch) != len(rhs_batch) or len(lhs_contract) != len(rhs_contract):
        raise ValueError("batch / contracting dimension lists differ in length")
    for a, b in zip(lhs_batch, rhs_batch):
        if lhs.shape[a] != rhs.shape[b]:
            raise ValueError("batch dimension sizes differ")
    for a, b in zip(lhs_contract, rhs_contract):
        if lhs.shape[a] != rhs.shape[b]:
            raise ValueError("contracting dimension sizes differ")
    lf = _free_dims(lhs.ndim, lhs_batch, lhs_contract)
    rf = _free_dims(rhs.ndim, rhs_batch, rhs_contract)
    bshape = [lhs.shape[d] for d in lhs_batch]
    ishape = [lhs.shape[d] for d in lf]
    jshape = [rhs.shape[d] for d in rf]
    cshape = [lhs.shape[d] for d in lhs_contract]
    G = int(np.prod(bshape, dtype=np.int64))
    I = int(np.prod(ishape, dtype=np.int64))
    J = int(np.prod(jshape, dtype=np.int64))
    C = int(np.prod(cshape, dtype=np.int64))
    a = np.transpose(lhs, list(lhs_batch) + lf + list(lhs_contract)).reshape(G, I, C)
    b = np.transpose(rhs, list(rhs_batch) + list(rhs_contract) + rf).reshape(G, C, J)
    out = np.matmul(a, b)
    return out.reshape(bshape + ishape + jshape)


def mask_beyond(x: np.ndarray, dim: int, valid: int) -> np.ndarray:
    """Select(Iota < valid, x, 0) along `dim` (Section 4.1, appendix Table 9)."""
    x = np.array(x, dtype=np.float64, copy=True)
    idx = [slice(None)] * x.ndim
    idx[dim] = slice(max(0, valid), None)
    x[tuple(idx)] = 0.0
    return x


def apply_fill(lhs: np.ndarray, lhs_batch: Sequence[int], free_dim: int,
               fill: Sequence[int]) -> np.ndarray:
    """Zero lhs rows at positions >= fill[g] of `free_dim` for batch entry g.

    The capacity dimension of the mixture-of-experts einsum (Section 5.4) may be
    only partly occupied; unoccupied slots take no part in the sum and their
    output rows are zero.  `fill` is indexed by the row-major flattened batch index.
    """
    lhs = np.array(lhs, dtype=np.float64, copy=True)
    bshape = [lhs.shape[d] for d in lhs_batch]
    for g, idx in enumerate(np.ndindex(*bshape)):
        sel = [slice(None)] * lhs.ndim
        for d, i in zip(lhs_batch, idx):
            sel[d] = i
        sel[free_dim] = slice(int(fill[g]), None)
        lhs[tuple(sel)] = 0.0
    return lhs


def shard_slices(mesh_shape, device_ids, global_shape, dims_mapping, partition_id):
    """Slice objects selecting partition p's valid region of a global tensor."""
    off, valid, shard = _bounds.shard_bounds(mesh_shape, device_ids, global_shape,
                                             dims_mapping, partition_id)
    return tuple(slice(o, o + v) for o, v in zip(off, valid)), off, valid, shard


def expected_out_shard(out_global: np.ndarray, mesh_shape, device_ids,
                       out_map, partition_id) -> np.ndarray:
    """What partition p's output shard must hold, padded with zeros to the
    static shard shape (pad content is the library's own guarantee; the paper
    leaves it arbitrary)."""
    sl, off, valid, shard = shard_slices(mesh_shape, device_ids, out_global.shape,
                                         out_map, partition_id)
    full = np.zeros(shard, dtype=np.float64)
    full[tuple(slice(0, v) for v in valid)] = out_global[sl]
    return full


def expected_partial(lhs: np.ndarray, rhs: np.ndarray, dims, mesh_shape, device_ids,
                     lhs_map, rhs_map, partition_id) -> np.ndarray:
    """Partial product of partition p when contracting dims are split: the dot
    of the operands with every position outside p's shard along *contracting*
    dimensions replaced by 0 (Section 4.1 masking); non-contracting and batch
    dimensions are left whole, to be sliced by the caller."""
    lhs_batch, rhs_batch, lhs_contract, rhs_contract = dims
    lo, lv, _ = _bounds.shard_bounds(mesh_shape, device_ids, lhs.shape, lhs_map, partition_id)
    ro, rv, _ = _bounds.shard_bounds(mesh_shape, device_ids, rhs.shape, rhs_map, partition_id)
    a = np.array(lhs, dtype=np.float64, copy=True)
    b = np.array(rhs, dtype=np.float64, copy=True)
    for d in lhs_contract:
        keep = np.zeros(a.shape[d], dtype=bool)
        keep[lo[d]:lo[d] + lv[d]] = True
        shape = [1] * a.ndim
        shape[d] = -1
        a = a * keep.reshape(shape)
    for d in rhs_contract:
        keep = np.zeros(b.shape[d], dtype=bool)
        keep[ro[d]:ro[d] + rv[d]] = True
        shape = [1] * b.ndim
        shape[d] = -1
        b = b * keep.reshape(shape)
    return dot_general(a, b, lhs_batch, rhs_batch, lhs_contract, rhs_contract)


def relu(x: np.ndarray) -> np.ndarray:
    """Elementwise max(x, 0) of Section 5.1's feed-forward layer; NaN stays NaN."""
    return np.maximum(x, 0.0)


def error_metrics(got: np.ndarray, ref: np.ndarray) -> Tuple[float, float]:
    """(max over elements of |got-ref| / (|ref|+1), relative Frobenius error)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    d = np.abs(got - ref)
    scaled = float(np.max(d / (np.abs(ref) + 1.0)))
    nr = float(np.linalg.norm(ref.ravel()))
    fro = float(np.linalg.norm((got - ref).ravel())) / nr if nr > 0 else float(np.linalg.norm((got - ref).ravel()))
    return scaled, fro
