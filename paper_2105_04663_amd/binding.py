"""ctypes binding of libgspmd.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

F32, BF16 = 0, 1
AXIS_UNUSED, AXIS_BATCH, AXIS_LHS_FREE, AXIS_RHS_FREE, AXIS_CONTRACTING, AXIS_CONTRACTING_SCATTER = range(6)
EPILOGUE_NONE, EPILOGUE_RELU = 0, 1
LAYOUT_LHS_K_MAJOR, LAYOUT_RHS_K_CONTIGUOUS = 1, 2
KERNEL_SCALAR, KERNEL_MFMA_STAGED, KERNEL_MFMA = 0, 1, 2

EXPORTED_SYMBOLS = (
    "gspmd_status_string", "gspmd_shard_bounds", "gspmd_classify_dot", "gspmd_dot_workspace_bytes",
    "gspmd_local_dot", "gspmd_grouped_dot", "gspmd_reduce_partials", "gspmd_shard_extract",
    "gspmd_shard_assemble", "gspmd_plan_dot", "gspmd_infer_out_sharding", "gspmd_reshard_workspace_bytes", "gspmd_reshard",
    "gspmd_compatible_operand_shardings", "gspmd_resharded_dot_workspace_bytes", "gspmd_resharded_dot",
    "gspmd_grouped_dot_noalloc", "gspmd_set_tile_timeline",
)
TILE_TIMELINE_WORDS = 8
NOALLOC_MAX_WORKSPACE_BYTES = 32 * 1024 * 1024


class GspmdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class _CMesh(C.Structure):
    _fields_ = [("rank", C.c_int32), ("shape", C.POINTER(C.c_int64)), ("device_ids", C.POINTER(C.c_int64))]


class _CSharding(C.Structure):
    _fields_ = [("rank", C.c_int32), ("global_shape", C.POINTER(C.c_int64)), ("dims_mapping", C.POINTER(C.c_int32))]


class _CDotDims(C.Structure):
    _fields_ = [("n_batch", C.c_int32), ("lhs_batch", C.POINTER(C.c_int32)), ("rhs_batch", C.POINTER(C.c_int32)),
                ("n_contract", C.c_int32), ("lhs_contract", C.POINTER(C.c_int32)), ("rhs_contract", C.POINTER(C.c_int32))]


class _CShardBuf(C.Structure):
    _fields_ = [("data", C.c_void_p), ("dtype", C.c_int32), ("row_stride", C.c_int64)]


class _CGemmDesc(C.Structure):
    _fields_ = [("a_offset", C.c_int64), ("b_offset", C.c_int64), ("c_offset", C.c_int64),
                ("lda", C.c_int64), ("ldb", C.c_int64), ("ldc", C.c_int64),
                ("m_valid", C.c_int32), ("n_valid", C.c_int32), ("k_valid", C.c_int32),
                ("m_static", C.c_int32), ("n_static", C.c_int32), ("layout", C.c_int32), ("kernel", C.c_int32),
                ("reserved", C.c_int32)]


_LIB = None


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgspmd.so")


def load_library():
    """Load libgspmd.so (built in-tree by paper_2105_04663_amd.build); raises if absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -m paper_2105_04663_amd.build` (no fallback exists)")
    lib = C.CDLL(path)
    lib.gspmd_status_string.restype = C.c_char_p
    lib.gspmd_status_string.argtypes = [C.c_int32]
    pm, ps, pd, pb = C.POINTER(_CMesh), C.POINTER(_CSharding), C.POINTER(_CDotDims), C.POINTER(_CShardBuf)
    pi64, pi32 = C.POINTER(C.c_int64), C.POINTER(C.c_int32)
    lib.gspmd_shard_bounds.argtypes = [pm, ps, C.c_int64, pi64, pi64, pi64]
    lib.gspmd_classify_dot.argtypes = [pm, pd, ps, ps, ps, pi32]
    lib.gspmd_dot_workspace_bytes.argtypes = [pm, pd, ps, ps, ps, C.c_int64, C.c_int32, pi64]
    lib.gspmd_local_dot.argtypes = [pm, pd, pb, ps, pb, ps, pb, ps, C.c_int64, pi64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
    lib.gspmd_grouped_dot.argtypes = [pm, pd, pb, ps, pb, ps, pb, ps, pi64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
    lib.gspmd_grouped_dot_noalloc.argtypes = [pm, pd, pb, ps, pb, ps, pb, ps, pi64, C.c_int32, C.c_void_p]
    lib.gspmd_reduce_partials.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p]
    lib.gspmd_shard_extract.argtypes = [pm, ps, C.c_int64, C.c_void_p, pb, C.c_uint32, C.c_void_p]
    lib.gspmd_shard_assemble.argtypes = [pm, ps, C.c_int64, pb, C.c_void_p, C.c_void_p]
    lib.gspmd_infer_out_sharding.argtypes = [pm, pd, ps, ps, pi32, pi64, pi32]
    lib.gspmd_reshard_workspace_bytes.argtypes = [pm, pi64]
    lib.gspmd_reshard.argtypes = [pm, ps, pb, ps, pb, C.c_void_p, C.c_int64, C.c_void_p]
    lib.gspmd_compatible_operand_shardings.argtypes = [pm, pd, ps, ps, ps, pi32, pi32]
    lib.gspmd_resharded_dot_workspace_bytes.argtypes = [pm, pd, ps, ps, ps, C.c_int32, pi64]
    lib.gspmd_resharded_dot.argtypes = [pm, pd, pb, ps, pb, ps, pb, ps, pi64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
    lib.gspmd_plan_dot.argtypes = [pm, pd, ps, ps, ps, C.c_int64, C.c_int64, C.c_int64, C.c_int64, pi64,
                                   C.POINTER(_CGemmDesc), C.c_int64, pi64]
    lib.gspmd_set_tile_timeline.argtypes = [C.c_void_p, C.c_int64]
    for name in EXPORTED_SYMBOLS[1:]:
        getattr(lib, name).restype = C.c_int32
    _LIB = lib
    return lib


def status_string(status: int) -> str:
    return load_library().gspmd_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise GspmdError(status, where)


def _i64(vals: Sequence[int]):
    return (C.c_int64 * max(1, len(vals)))(*[int(v) for v in vals])


def _i32(vals: Sequence[int]):
    return (C.c_int32 * max(1, len(vals)))(*[int(v) for v in vals])


@dataclass
class Mesh:
    """Device mesh: shape and the row-major tensor of partition ids."""
    shape: Tuple[int, ...]
    device_ids: Tuple[int, ...]

    def _c(self):
        self._keep = (_i64(self.shape), _i64(self.device_ids))
        return _CMesh(len(self.shape), self._keep[0], self._keep[1])

    @property
    def n_partitions(self) -> int:
        n = 1
        for s in self.shape:
            n *= int(s)
        return n


@dataclass
class Sharding:
    """mesh_split annotation: unpartitioned shape and dims_mapping (-1 = not split)."""
    global_shape: Tuple[int, ...]
    dims_mapping: Tuple[int, ...]

    def _c(self):
        self._keep = (_i64(self.global_shape), _i32(self.dims_mapping))
        rank = len(self.global_shape) if len(self.global_shape) == len(self.dims_mapping) else -1
        return _CSharding(rank, self._keep[0], self._keep[1])


@dataclass
class DotDims:
    lhs_batch: Tuple[int, ...]
    rhs_batch: Tuple[int, ...]
    lhs_contract: Tuple[int, ...]
    rhs_contract: Tuple[int, ...]

    def _c(self):
        self._keep = (_i32(self.lhs_batch), _i32(self.rhs_batch), _i32(self.lhs_contract), _i32(self.rhs_contract))
        nb = len(self.lhs_batch) if len(self.lhs_batch) == len(self.rhs_batch) else -1
        nc = len(self.lhs_contract) if len(self.lhs_contract) == len(self.rhs_contract) else -1
        return _CDotDims(nb, self._keep[0], self._keep[1], nc, self._keep[2], self._keep[3])


@dataclass
class ShardBuf:
    """A shard in device memory: raw pointer, dtype code and row stride in elements (0 = dense)."""
    data: int
    dtype: int
    row_stride: int = 0

    @staticmethod
    def of(tensor, row_stride: int = 0) -> "ShardBuf":
        """Describe a torch tensor's storage (no copy); bf16 and float32 only."""
        import torch
        if tensor.dtype == torch.bfloat16:
            dt = BF16
        elif tensor.dtype == torch.float32:
            dt = F32
        else:
            raise TypeError("shard buffers are bfloat16 or float32")
        return ShardBuf(tensor.data_ptr(), dt, row_stride)

    def _c(self):
        return _CShardBuf(C.c_void_p(self.data), self.dtype, self.row_stride)


def _bufs(bufs: Sequence[ShardBuf]):
    arr = (_CShardBuf * max(1, len(bufs)))()
    for i, b in enumerate(bufs):
        arr[i] = b._c()
    return arr


def shard_bounds(mesh: Mesh, sharding: Sharding, partition_id: int):
    """(offset, valid_len, shard_size) tuples per tensor dimension."""
    r = max(1, len(sharding.global_shape))
    off, valid, shard = (C.c_int64 * r)(), (C.c_int64 * r)(), (C.c_int64 * r)()
    m, s = mesh._c(), sharding._c()
    _check(load_library().gspmd_shard_bounds(C.byref(m), C.byref(s), int(partition_id), off, valid, shard), "gspmd_shard_bounds")
    n = len(sharding.global_shape)
    return tuple(off[:n]), tuple(valid[:n]), tuple(shard[:n])


def classify_dot(mesh: Mesh, dims: DotDims, lhs_sh: Sharding, rhs_sh: Sharding, out_sh: Sharding) -> Tuple[int, ...]:
    cls = (C.c_int32 * max(1, len(mesh.shape)))()
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    _check(load_library().gspmd_classify_dot(C.byref(m), C.byref(d), C.byref(a), C.byref(b), C.byref(o), cls), "gspmd_classify_dot")
    return tuple(cls[:len(mesh.shape)])


def dot_workspace_bytes(mesh: Mesh, dims: DotDims, lhs_sh: Sharding, rhs_sh: Sharding, out_sh: Sharding,
                        partition_id: int = -1, has_fill: bool = False) -> int:
    n = C.c_int64(0)
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    _check(load_library().gspmd_dot_workspace_bytes(C.byref(m), C.byref(d), C.byref(a), C.byref(b), C.byref(o),
                                                    int(partition_id), int(has_fill), C.byref(n)), "gspmd_dot_workspace_bytes")
    return int(n.value)


def infer_out_sharding(mesh: Mesh, dims: DotDims, lhs_sh: Sharding, rhs_sh: Sharding) -> Sharding:
    """Output sharding merged from the operand shardings (Section 3.5)."""
    m, d, a, b = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c()
    cap = len(lhs_sh.global_shape) + len(rhs_sh.global_shape) + 1
    mapping, shape, rank = (C.c_int32 * cap)(), (C.c_int64 * cap)(), C.c_int32(0)
    _check(load_library().gspmd_infer_out_sharding(C.byref(m), C.byref(d), C.byref(a), C.byref(b), mapping, shape,
                                                   C.byref(rank)), "gspmd_infer_out_sharding")
    return Sharding(tuple(shape[:rank.value]), tuple(mapping[:rank.value]))


def plan_dot(mesh: Mesh, dims: DotDims, lhs_sh: Sharding, rhs_sh: Sharding, out_sh: Sharding, partition_id: int,
             lhs_row_stride: int = 0, rhs_row_stride: int = 0, out_row_stride: int = 0, lhs_fill=None) -> List[dict]:
    """The strided GEMMs partition `partition_id`'s local Dot is lowered to (host only)."""
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    n = C.c_int64(0)
    lib = load_library()
    args = (C.byref(m), C.byref(d), C.byref(a), C.byref(b), C.byref(o), int(lhs_row_stride), int(rhs_row_stride),
            int(out_row_stride), int(partition_id), _fill(lhs_fill))
    _check(lib.gspmd_plan_dot(*args, None, 0, C.byref(n)), "gspmd_plan_dot")
    arr = (_CGemmDesc * max(1, n.value))()
    _check(lib.gspmd_plan_dot(*args, arr, n.value, C.byref(n)), "gspmd_plan_dot")
    return [{f: getattr(arr[i], f) for f, _ in _CGemmDesc._fields_} for i in range(n.value)]


def _fill(fill):
    if fill is None:
        return None
    return _i64([int(x) for x in fill])


def local_dot(mesh: Mesh, dims: DotDims, lhs: ShardBuf, lhs_sh: Sharding, rhs: ShardBuf, rhs_sh: Sharding,
              out: ShardBuf, out_sh: Sharding, partition_id: int, lhs_fill=None,
              workspace: int = 0, workspace_bytes: int = 0, stream: int = 0, epilogue: int = EPILOGUE_NONE) -> None:
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    la, rb, ob = lhs._c(), rhs._c(), out._c()
    _check(load_library().gspmd_local_dot(C.byref(m), C.byref(d), C.byref(la), C.byref(a), C.byref(rb), C.byref(b),
                                          C.byref(ob), C.byref(o), int(partition_id), _fill(lhs_fill), int(epilogue),
                                          C.c_void_p(workspace), int(workspace_bytes), C.c_void_p(stream)), "gspmd_local_dot")


def grouped_dot(mesh: Mesh, dims: DotDims, lhs_shards: Sequence[ShardBuf], lhs_sh: Sharding,
                rhs_shards: Sequence[ShardBuf], rhs_sh: Sharding, out_shards: Sequence[ShardBuf], out_sh: Sharding,
                lhs_fill=None, workspace: int = 0, workspace_bytes: int = 0, stream: int = 0,
                epilogue: int = EPILOGUE_NONE) -> None:
    P = mesh.n_partitions
    if not (len(lhs_shards) == len(rhs_shards) == len(out_shards) == P):
        raise ValueError("one shard buffer per partition is required")
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    _check(load_library().gspmd_grouped_dot(C.byref(m), C.byref(d), _bufs(lhs_shards), C.byref(a), _bufs(rhs_shards), C.byref(b),
                                            _bufs(out_shards), C.byref(o), _fill(lhs_fill), int(epilogue),
                                            C.c_void_p(workspace), int(workspace_bytes), C.c_void_p(stream)), "gspmd_grouped_dot")


def grouped_dot_noalloc(mesh: Mesh, dims: DotDims, lhs_shards: Sequence[ShardBuf], lhs_sh: Sharding,
                        rhs_shards: Sequence[ShardBuf], rhs_sh: Sharding, out_shards: Sequence[ShardBuf], out_sh: Sharding,
                        lhs_fill=None, stream: int = 0, epilogue: int = EPILOGUE_NONE) -> None:
    """grouped_dot with the library's static workspace (no workspace argument, nothing allocated)."""
    P = mesh.n_partitions
    if not (len(lhs_shards) == len(rhs_shards) == len(out_shards) == P):
        raise ValueError("one shard buffer per partition is required")
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    _check(load_library().gspmd_grouped_dot_noalloc(C.byref(m), C.byref(d), _bufs(lhs_shards), C.byref(a), _bufs(rhs_shards),
                                                    C.byref(b), _bufs(out_shards), C.byref(o), _fill(lhs_fill), int(epilogue),
                                                    C.c_void_p(stream)), "gspmd_grouped_dot_noalloc")


def reshard_workspace_bytes(mesh: Mesh) -> int:
    m, n = mesh._c(), C.c_int64(0)
    _check(load_library().gspmd_reshard_workspace_bytes(C.byref(m), C.byref(n)), "gspmd_reshard_workspace_bytes")
    return n.value


def reshard(mesh: Mesh, src_sh: Sharding, src_shards: Sequence[ShardBuf], dst_sh: Sharding, dst_shards: Sequence[ShardBuf],
            workspace: int = 0, workspace_bytes: int = 0, stream: int = 0) -> None:
    P = mesh.n_partitions
    if not (len(src_shards) == len(dst_shards) == P):
        raise ValueError("one shard buffer per partition is required")
    m, a, b = mesh._c(), src_sh._c(), dst_sh._c()
    _check(load_library().gspmd_reshard(C.byref(m), C.byref(a), _bufs(src_shards), C.byref(b), _bufs(dst_shards),
                                        C.c_void_p(workspace), int(workspace_bytes), C.c_void_p(stream)), "gspmd_reshard")


def compatible_operand_shardings(mesh: Mesh, dims: DotDims, lhs_sh: Sharding, rhs_sh: Sharding, out_sh: Sharding):
    """(lhs mapping, rhs mapping) the Dot can consume without communication under `out_sh` (host only)."""
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    lm, rm = (C.c_int32 * max(1, a.rank))(), (C.c_int32 * max(1, b.rank))()
    _check(load_library().gspmd_compatible_operand_shardings(C.byref(m), C.byref(d), C.byref(a), C.byref(b), C.byref(o), lm, rm),
           "gspmd_compatible_operand_shardings")
    return tuple(lm[i] for i in range(a.rank)), tuple(rm[i] for i in range(b.rank))


def resharded_dot_workspace_bytes(mesh: Mesh, dims: DotDims, lhs_sh: Sharding, rhs_sh: Sharding, out_sh: Sharding,
                                  in_dtype: int) -> int:
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    n = C.c_int64(0)
    _check(load_library().gspmd_resharded_dot_workspace_bytes(C.byref(m), C.byref(d), C.byref(a), C.byref(b), C.byref(o),
                                                              int(in_dtype), C.byref(n)), "gspmd_resharded_dot_workspace_bytes")
    return n.value


def resharded_dot(mesh: Mesh, dims: DotDims, lhs_shards: Sequence[ShardBuf], lhs_sh: Sharding,
                  rhs_shards: Sequence[ShardBuf], rhs_sh: Sharding, out_shards: Sequence[ShardBuf], out_sh: Sharding,
                  lhs_fill=None, workspace: int = 0, workspace_bytes: int = 0, stream: int = 0,
                  epilogue: int = EPILOGUE_NONE) -> None:
    P = mesh.n_partitions
    if not (len(lhs_shards) == len(rhs_shards) == len(out_shards) == P):
        raise ValueError("one shard buffer per partition is required")
    m, d, a, b, o = mesh._c(), dims._c(), lhs_sh._c(), rhs_sh._c(), out_sh._c()
    _check(load_library().gspmd_resharded_dot(C.byref(m), C.byref(d), _bufs(lhs_shards), C.byref(a), _bufs(rhs_shards), C.byref(b),
                                              _bufs(out_shards), C.byref(o), _fill(lhs_fill), int(epilogue),
                                              C.c_void_p(workspace), int(workspace_bytes), C.c_void_p(stream)), "gspmd_resharded_dot")


def reduce_partials(partials: Sequence[int], n_elems: int, out: int, out_dtype: int, stream: int = 0) -> None:
    arr = (C.c_void_p * max(1, len(partials)))(*[C.c_void_p(int(p)) for p in partials])
    _check(load_library().gspmd_reduce_partials(arr, len(partials), int(n_elems), C.c_void_p(out), int(out_dtype),
                                                C.c_void_p(stream)), "gspmd_reduce_partials")


def shard_extract(mesh: Mesh, sharding: Sharding, partition_id: int, global_data: int, shard: ShardBuf,
                  pad_bits: int = 0, stream: int = 0) -> None:
    m, s, b = mesh._c(), sharding._c(), shard._c()
    _check(load_library().gspmd_shard_extract(C.byref(m), C.byref(s), int(partition_id), C.c_void_p(global_data),
                                              C.byref(b), C.c_uint32(pad_bits & 0xFFFFFFFF), C.c_void_p(stream)), "gspmd_shard_extract")


def shard_assemble(mesh: Mesh, sharding: Sharding, partition_id: int, shard: ShardBuf, global_data: int,
                   stream: int = 0) -> None:
    m, s, b = mesh._c(), sharding._c(), shard._c()
    _check(load_library().gspmd_shard_assemble(C.byref(m), C.byref(s), int(partition_id), C.byref(b),
                                               C.c_void_p(global_data), C.c_void_p(stream)), "gspmd_shard_assemble")


def set_tile_timeline(device_records: int, n_records: int) -> None:
    """gspmd_set_tile_timeline: device_records = address of n_records * 64 bytes of cleared device memory, or 0 to switch off."""
    _check(load_library().gspmd_set_tile_timeline(C.c_void_p(int(device_records) or None), int(n_records)), "gspmd_set_tile_timeline")
