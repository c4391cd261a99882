"""Seeded synthetic inputs for the GSPMD per-partition einsum path.

This module only *draws numbers and describes shapes*.  It holds none of the
method's arithmetic (no shard bounds, no contraction, no masking): both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so
that the two sides see bit-identical operands while sharing no other code.

The shapes stand in for the paper's workloads: the Transformer feed-forward
einsum BSM,MH->BSH with M = 8192 (Section 5.1, Table 1 "2D finalized" row), the
mixture-of-experts einsum ECM,EMH->ECH with H = 32768 (Section 5.4/5.5), a
contracting-dimension split (Section 5.1, "2D Attempt 1") and a nested 2-D
mesh (Section 4.4).  Values are N(0,1) activations and N(0, 0.02^2) weights
rounded to bfloat16, or U(-1,1) float32 for the tiny case.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 210504663 * 100


def seed_for(cfg: int, t: int) -> int:
    """Seed of tensor `t` (0 lhs, 1 rhs, 2 fill counts) of config `cfg`."""
    return SEED_BASE + 10 * cfg + t


# ----------------------------------------------------------------------------
# bfloat16 as raw bits.  Inputs are *defined* as bf16 values, so producing the
# bit pattern is part of drawing the input, not of the method under test.
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits.

    NaN is not expected in synthetic inputs and is not special-cased.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bits to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bits to float64."""
    return bf16_bits_to_f32(b).astype(np.float64)


def draw_normal_bf16(seed: int, shape: Sequence[int], sigma: float = 1.0,
                     chunk: int = 1 << 24) -> np.ndarray:
    """N(0, sigma^2) float32 draws rounded to bf16 bits; chunked to bound RAM."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    s = np.float32(sigma)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        v = rng.standard_normal(hi - lo, dtype=np.float32)
        if sigma != 1.0:
            v *= s
        out[lo:hi] = f32_to_bf16_bits(v)
    return out.reshape(tuple(shape))


def draw_uniform_f32(seed: int, shape: Sequence[int], lo: float = -1.0,
                     hi: float = 1.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.uniform(lo, hi, size=tuple(shape)).astype(np.float32)


def draw_small_int_bf16(seed: int, shape: Sequence[int], lo: int = -8,
                        hi: int = 8) -> np.ndarray:
    """Integers in [lo, hi] as bf16 bits (all exactly representable)."""
    rng = np.random.default_rng(seed)
    v = rng.integers(lo, hi + 1, size=tuple(shape)).astype(np.float32)
    return f32_to_bf16_bits(v)


def draw_fill_counts(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """Per-expert number of occupied capacity slots, uniform on [lo, hi]."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=n).astype(np.int64)


# ----------------------------------------------------------------------------
# Workload descriptions
# ----------------------------------------------------------------------------
@dataclass
class DotWorkload:
    """One sharded dot_general problem: global shapes, mesh and mappings."""
    name: str
    cfg: int
    dtype: str                       # "bf16" or "f32"
    out_dtype: str                   # "bf16" or "f32"
    lhs_shape: Tuple[int, ...]
    rhs_shape: Tuple[int, ...]
    lhs_batch: Tuple[int, ...]
    rhs_batch: Tuple[int, ...]
    lhs_contract: Tuple[int, ...]
    rhs_contract: Tuple[int, ...]
    mesh_shape: Tuple[int, ...]
    device_ids: Tuple[int, ...]      # row-major device-ID tensor
    lhs_map: Tuple[int, ...]
    rhs_map: Tuple[int, ...]
    out_map: Tuple[int, ...]
    lhs_sigma: float = 1.0
    rhs_sigma: float = 0.02
    fill_range: Optional[Tuple[int, int]] = None   # MoE capacity fill
    einsum: str = ""

    @property
    def out_shape(self) -> Tuple[int, ...]:
        lb, rb = self.lhs_batch, self.rhs_batch
        lf = [d for d in range(len(self.lhs_shape))
              if d not in lb and d not in self.lhs_contract]
        rf = [d for d in range(len(self.rhs_shape))
              if d not in rb and d not in self.rhs_contract]
        return tuple([self.lhs_shape[d] for d in lb]
                     + [self.lhs_shape[d] for d in lf]
                     + [self.rhs_shape[d] for d in rf])

    @property
    def n_partitions(self) -> int:
        return int(np.prod(self.mesh_shape))

    def draw_lhs(self) -> np.ndarray:
        """bf16 bits (uint16) or float32 values of the global lhs tensor."""
        if self.dtype == "f32":
            return draw_uniform_f32(seed_for(self.cfg, 0), self.lhs_shape)
        x = draw_normal_bf16(seed_for(self.cfg, 0), self.lhs_shape, self.lhs_sigma)
        fill = self.draw_fill()
        if fill is not None:
            # capacity slots beyond the fill count hold no token: zero rows
            for e in range(self.lhs_shape[0]):
                x[e, int(fill[e]):] = 0
        return x

    def draw_rhs(self) -> np.ndarray:
        if self.dtype == "f32":
            return draw_uniform_f32(seed_for(self.cfg, 1), self.rhs_shape)
        return draw_normal_bf16(seed_for(self.cfg, 1), self.rhs_shape, self.rhs_sigma)

    def draw_fill(self) -> Optional[np.ndarray]:
        if self.fill_range is None:
            return None
        return draw_fill_counts(seed_for(self.cfg, 2), self.lhs_shape[0],
                                self.fill_range[0], self.fill_range[1])

    def useful_flops(self, fill: Optional[np.ndarray] = None) -> float:
        """2 * (valid output elements) * K, counting only occupied MoE rows."""
        k = 1
        for d in self.lhs_contract:
            k *= self.lhs_shape[d]
        out = self.out_shape
        if self.fill_range is not None:
            # the capacity dimension (lhs dim 1) counts with its fill, whether it is a row or a contracting dimension
            if fill is None:
                fill = self.draw_fill()
            rest = float(np.prod(out[1:])) * k / self.lhs_shape[1]
            return 2.0 * float(np.sum(fill)) * rest
        return 2.0 * float(np.prod(out)) * k

    def padded_flops(self) -> float:
        """2 * (output elements) * K over the STATIC shard shapes: every split dimension rounded up to a multiple of its
        mesh dimension, capacity slots counted whether occupied or not -- the convention of a profiler that counts
        padded compute as valid compute (Section 5.2)."""
        def padded(size: int, mesh_dim: int) -> int:
            n = self.mesh_shape[mesh_dim] if mesh_dim >= 0 else 1
            return n * (-(-size // n))
        k = 1
        for d in self.lhs_contract:
            k *= padded(self.lhs_shape[d], self.lhs_map[d])
        out = 1
        for size, mesh_dim in zip(self.out_shape, self.out_map):
            out *= padded(size, mesh_dim)
        return 2.0 * float(out) * float(k)


def _ids(n: int) -> Tuple[int, ...]:
    return tuple(range(n))


def tiny_1d() -> DotWorkload:
    """Config 1: A[8,64] x B[64,90] f32, N split over 4 partitions (23,23,23,21)."""
    return DotWorkload(
        name="tiny_1d_matmul", cfg=1, dtype="f32", out_dtype="f32",
        lhs_shape=(8, 64), rhs_shape=(64, 90),
        lhs_batch=(), rhs_batch=(), lhs_contract=(1,), rhs_contract=(0,),
        mesh_shape=(4,), device_ids=_ids(4),
        lhs_map=(-1, -1), rhs_map=(-1, 0), out_map=(-1, 0), einsum="mk,kn->mn")


def ffn(B: int = 8, S: int = 2048, M: int = 8192, H: int = 8192) -> DotWorkload:
    """Config 2: one device's share of BSM,MH->BSH on a 2-D mesh (1 partition)."""
    return DotWorkload(
        name="ffn_bsm_mh", cfg=2, dtype="bf16", out_dtype="bf16",
        lhs_shape=(B, S, M), rhs_shape=(M, H),
        lhs_batch=(), rhs_batch=(), lhs_contract=(2,), rhs_contract=(0,),
        mesh_shape=(1, 1), device_ids=(0,),
        lhs_map=(0, -1, -1), rhs_map=(-1, 1), out_map=(0, -1, 1),
        einsum="BSM,MH->BSH")


def ksplit(M: int = 4096, K: int = 16384, N: int = 8192, P: int = 4) -> DotWorkload:
    """Config 3: contracting dim split over P partitions; fp32 partials."""
    return DotWorkload(
        name="ksplit_matmul", cfg=3, dtype="bf16", out_dtype="f32",
        lhs_shape=(M, K), rhs_shape=(K, N),
        lhs_batch=(), rhs_batch=(), lhs_contract=(1,), rhs_contract=(0,),
        mesh_shape=(P,), device_ids=_ids(P),
        lhs_map=(-1, 0), rhs_map=(0, -1), out_map=(-1, -1), einsum="mk,kn->mn")


def moe(E: int = 4, C: int = 1024, M: int = 8192, H: int = 32768,
        fill_lo: Optional[int] = None) -> DotWorkload:
    """Config 4: one device's share of ECM,EMH->ECH; per-expert fill counts."""
    lo = C // 2 if fill_lo is None else fill_lo
    return DotWorkload(
        name="moe_ecm_emh", cfg=4, dtype="bf16", out_dtype="bf16",
        lhs_shape=(E, C, M), rhs_shape=(E, M, H),
        lhs_batch=(0,), rhs_batch=(0,), lhs_contract=(2,), rhs_contract=(1,),
        mesh_shape=(1,), device_ids=(0,),
        lhs_map=(0, -1, -1), rhs_map=(0, -1, -1), out_map=(0, -1, -1),
        fill_range=(lo, C), einsum="ECM,EMH->ECH")


def mesh2d(M: int = 6000, K: int = 12288, N: int = 10000, X: int = 4, Y: int = 8,
           cfg: int = 5, device_ids: Optional[Sequence[int]] = None) -> DotWorkload:
    """Config 5: rows on mesh axis 0, columns on mesh axis 1; X*Y partitions."""
    ids = _ids(X * Y) if device_ids is None else tuple(int(i) for i in device_ids)
    return DotWorkload(
        name="mesh2d_grouped", cfg=cfg, dtype="bf16", out_dtype="bf16",
        lhs_shape=(M, K), rhs_shape=(K, N),
        lhs_batch=(), rhs_batch=(), lhs_contract=(1,), rhs_contract=(0,),
        mesh_shape=(X, Y), device_ids=ids,
        lhs_map=(0, -1), rhs_map=(-1, 1), out_map=(0, 1), einsum="mk,kn->mn")


def mesh2d_uneven() -> DotWorkload:
    """Sibling of config 5 whose dims do not divide: 5998/4 and 9999/8."""
    return mesh2d(M=5998, K=12288, N=9999, cfg=6)




def ffn_second(B: int = 8, S: int = 2048, H: int = 32768, M: int = 8192, Y: int = 4, scatter: bool = False) -> DotWorkload:
    """Second feed-forward einsum BSH,HM->BSM with H split over Y partitions (Section 5.1, Table 1): every partition
    contracts its H slice and holds a partial BSM that the AllReduce sums; with `scatter` the output's M is split over
    Y as well ("2D finalized" of Table 1) and the sum is a ReduceScatter."""
    return DotWorkload(
        name="ffn_bsh_hm_rs" if scatter else "ffn_bsh_hm", cfg=7, dtype="bf16", out_dtype="bf16",
        lhs_shape=(B, S, H), rhs_shape=(H, M),
        lhs_batch=(), rhs_batch=(), lhs_contract=(2,), rhs_contract=(0,),
        mesh_shape=(Y,), device_ids=_ids(Y),
        lhs_map=(-1, -1, 0), rhs_map=(0, -1), out_map=(-1, -1, 0 if scatter else -1), einsum="BSH,HM->BSM")


def moe_second(E: int = 4, C: int = 1024, H: int = 32768, M: int = 8192) -> DotWorkload:
    """Second expert einsum ECH,EHM->ECM on one device's share (Section 5.4), with per-expert fill counts."""
    return DotWorkload(
        name="moe_ech_ehm", cfg=8, dtype="bf16", out_dtype="bf16",
        lhs_shape=(E, C, H), rhs_shape=(E, H, M),
        lhs_batch=(0,), rhs_batch=(0,), lhs_contract=(2,), rhs_contract=(1,),
        mesh_shape=(1,), device_ids=(0,),
        lhs_map=(0, -1, -1), rhs_map=(0, -1, -1), out_map=(0, -1, -1),
        fill_range=(C // 2, C), einsum="ECH,EHM->ECM")


def ffn_wgrad(B: int = 8, S: int = 2048, M: int = 8192, H: int = 8192, X: int = 1, Y: int = 1) -> DotWorkload:
    """Weight gradient of the first feed-forward einsum, BSM,BSH->MH: the token dims contract, so both operands are
    K-major.  With B split over X partitions (data parallelism) every partition holds a partial gradient that the
    AllReduce / ReduceScatter over X sums (Section 3.2's backward pass); H stays split over Y.  X = Y = 1 is one
    device's share of the 2-D mesh."""
    return DotWorkload(
        name="ffn_wgrad_bsm_bsh", cfg=9, dtype="bf16", out_dtype="bf16",
        lhs_shape=(B, S, M), rhs_shape=(B, S, H),
        lhs_batch=(), rhs_batch=(), lhs_contract=(0, 1), rhs_contract=(0, 1),
        mesh_shape=(X, Y), device_ids=_ids(X * Y),
        lhs_map=(0, -1, -1), rhs_map=(0, -1, 1), out_map=(-1, 1), rhs_sigma=1.0, einsum="BSM,BSH->MH")


def ffn_dgrad(B: int = 8, S: int = 2048, H: int = 8192, M: int = 8192, X: int = 1, Y: int = 1) -> DotWorkload:
    """Input gradient of the first feed-forward einsum, BSH,MH->BSM: H contracts and is the last dimension of both
    operands (both K-contiguous).  B split over X (lhs non-contracting), H over Y (contracting: partial sums)."""
    return DotWorkload(
        name="ffn_dgrad_bsh_mh", cfg=10, dtype="bf16", out_dtype="bf16",
        lhs_shape=(B, S, H), rhs_shape=(M, H),
        lhs_batch=(), rhs_batch=(), lhs_contract=(2,), rhs_contract=(1,),
        mesh_shape=(X, Y), device_ids=_ids(X * Y),
        lhs_map=(0, -1, 1), rhs_map=(-1, 1), out_map=(0, -1, -1), einsum="BSH,MH->BSM")


def attn_qkv(B: int = 8, S: int = 2048, M: int = 8192, N: int = 32, D: int = 256, X: int = 1, Y: int = 1) -> DotWorkload:
    """Attention input projection BSM,MND->BSND (Table 1: W_Q, W_K, W_V of shape MND): B split over X, the heads N over
    Y; the rhs has two non-contracting dimensions.  Defaults are one device's share (N = 128 heads / 4)."""
    return DotWorkload(
        name="attn_bsm_mnd", cfg=11, dtype="bf16", out_dtype="bf16",
        lhs_shape=(B, S, M), rhs_shape=(M, N, D),
        lhs_batch=(), rhs_batch=(), lhs_contract=(2,), rhs_contract=(0,),
        mesh_shape=(X, Y), device_ids=_ids(X * Y),
        lhs_map=(0, -1, -1), rhs_map=(-1, 1, -1), out_map=(0, -1, 1, -1), einsum="BSM,MND->BSND")


def attn_out(B: int = 8, S: int = 2048, N: int = 32, D: int = 256, M: int = 8192, X: int = 1, Y: int = 1,
             scatter: bool = False) -> DotWorkload:
    """Attention output projection BSND,NDM->BSM (Table 1: W_O of shape NDM): two contracting dimensions, the heads N
    split over Y, so every partition holds a partial BSM (AllReduce, or ReduceScatter with M split over Y as well)."""
    return DotWorkload(
        name="attn_bsnd_ndm", cfg=12, dtype="bf16", out_dtype="bf16",
        lhs_shape=(B, S, N, D), rhs_shape=(N, D, M),
        lhs_batch=(), rhs_batch=(), lhs_contract=(2, 3), rhs_contract=(0, 1),
        mesh_shape=(X, Y), device_ids=_ids(X * Y),
        lhs_map=(0, -1, 1, -1), rhs_map=(1, -1, -1), out_map=(0, -1, 1 if scatter else -1), einsum="BSND,NDM->BSM")


def moe_wgrad(E: int = 4, C: int = 1024, M: int = 8192, H: int = 32768) -> DotWorkload:
    """Weight gradient of the first expert einsum, ECM,ECH->EMH: the capacity slots contract (both operands K-major),
    so the per-expert fill count limits K instead of the rows."""
    return DotWorkload(
        name="moe_wgrad_ecm_ech", cfg=13, dtype="bf16", out_dtype="bf16",
        lhs_shape=(E, C, M), rhs_shape=(E, C, H),
        lhs_batch=(0,), rhs_batch=(0,), lhs_contract=(1,), rhs_contract=(1,),
        mesh_shape=(1,), device_ids=(0,),
        lhs_map=(0, -1, -1), rhs_map=(0, -1, -1), out_map=(0, -1, -1), rhs_sigma=1.0,
        fill_range=(C // 2, C), einsum="ECM,ECH->EMH")


def all_configs() -> List[DotWorkload]:
    return [tiny_1d(), ffn(), ksplit(), moe(), mesh2d()]
