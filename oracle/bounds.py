"""CPU oracle: where a partition's shard sits in the unpartitioned tensor.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
it exists so that tests, the smoke check and the bench's cpu_baseline leg have
an independent statement of what the library must return.  It shares no code
with the HIP/C++ library.

What it states (all integer, exact):

* Section 3.1: a device mesh is a row-major tensor of device ids; `dims_mapping[i]`
  names the mesh dimension that tensor dimension i is split over, or -1.  A
  device owns the tile whose position equals the device's position in the mesh.
* Section 3.5 ("Merging compatible shardings"): Offset(S, d, i) is the position
  of device d's shard in dimension i of the unpartitioned shape.
* Section 4.1 ("Static shapes"): every partition has the same static shard size,
  the dimension rounded up to a multiple of the partition count and divided by
  it, i.e. ceil(D / n).  Section 4.3 keeps padding on the high side, so only
  trailing partitions are short; the worked reshape example there ((3,2) split
  two ways has partition shape (2,2)) fixes the ceil rule.

Readings where the paper is silent: the offset is coord * shard without
clamping (a pure function of the partition id), and a partition that lies
wholly in the padding has valid length 0.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def mesh_coords(mesh_shape: Sequence[int], device_ids: Sequence[int],
                partition_id: int) -> Tuple[int, ...]:
    """Position of `partition_id` in the row-major device-ID tensor (Section 3.1)."""
    total = 1
    for s in mesh_shape:
        if s <= 0:
            raise ValueError("mesh dimension must be positive")
        total *= s
    if len(device_ids) != total:
        raise ValueError("device_ids must have prod(mesh_shape) entries")
    if sorted(device_ids) != list(range(total)):
        raise ValueError("device_ids must be a permutation of 0..P-1")
    where = [i for i, d in enumerate(device_ids) if d == partition_id]
    if len(where) != 1:
        raise ValueError("partition id not in mesh")
    lin = where[0]
    coords: List[int] = []
    for s in reversed(list(mesh_shape)):
        coords.append(lin % s)
        lin //= s
    return tuple(reversed(coords))


def shard_bounds(mesh_shape: Sequence[int], device_ids: Sequence[int],
                 global_shape: Sequence[int], dims_mapping: Sequence[int],
                 partition_id: int):
    """(offset, valid_len, shard_size) per tensor dimension for one partition.

    Offset(S, d, i) of Section 3.5 with the static ceil-sized shards of
    Section 4.1; unmapped dimensions are whole (offset 0, valid = size).
    """
    if len(global_shape) != len(dims_mapping):
        raise ValueError("dims_mapping rank differs from tensor rank")
    used = [a for a in dims_mapping if a != -1]
    if any(a < 0 or a >= len(mesh_shape) for a in used):
        raise ValueError("mesh dimension out of range")
    if len(set(used)) != len(used):
        raise ValueError("a mesh dimension may appear at most once")
    coords = mesh_coords(mesh_shape, device_ids, partition_id)
    offset, valid, shard = [], [], []
    for size, axis in zip(global_shape, dims_mapping):
        if axis == -1:
            offset.append(0)
            valid.append(size)
            shard.append(size)
            continue
        n = mesh_shape[axis]
        per = -(-size // n)                 # ceil(size / n)
        off = coords[axis] * per
        offset.append(off)
        valid.append(max(0, min(per, size - off)))
        shard.append(per)
    return tuple(offset), tuple(valid), tuple(shard)


def is_merged_sharding(mesh_shape, device_ids, out_shape, out_map, inherited) -> bool:
    """Whether `out_map` is a merged sharding in the sense of Section 3.5.

    `inherited` lists (out_dim, operand_shape, operand_map, operand_dim): out dimension out_dim comes from that
    operand dimension.  The definition: for every device d and every *sharded* operand dimension i,
    Offset(S, d, i) == Offset(S_operand, d, i); and S splits no dimension the operands do not split.
    """
    total = 1
    for s in mesh_shape:
        total *= s
    sharded_out = set()
    for out_dim, op_shape, op_map, op_dim in inherited:
        if op_map[op_dim] == -1 or mesh_shape[op_map[op_dim]] == 1:
            continue
        sharded_out.add(out_dim)
        for d in range(total):
            o_off, _, _ = shard_bounds(mesh_shape, device_ids, out_shape, out_map, d)
            p_off, _, _ = shard_bounds(mesh_shape, device_ids, op_shape, op_map, d)
            if o_off[out_dim] != p_off[op_dim]:
                return False
    for i, a in enumerate(out_map):
        if a != -1 and mesh_shape[a] > 1 and i not in sharded_out:
            return False
    return True
