// Device kernels that are not MFMA-shaped: the any-layout fallback contraction (fp32 inputs,
// or bf16 inputs whose pointers/strides do not allow 16-byte loads), the K-partial sum and the
// shard <-> global copies.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace gspmd {

typedef uint16_t bf16_bits;

__device__ __forceinline__ float bf16_to_float(bf16_bits b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round-to-nearest-even; NaN stays NaN (quiet bit forced so the payload cannot round to Inf)
__device__ __forceinline__ bf16_bits float_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_bits>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_bits>(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_as_float(const T* p);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<bf16_bits>(const bf16_bits* p) { return bf16_to_float(*p); }

template <typename T> __device__ __forceinline__ void store_from_float(T* p, float v);
template <> __device__ __forceinline__ void store_from_float<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_float<bf16_bits>(bf16_bits* p, float v) { *p = float_to_bf16(v); }

// 16-byte accesses with the non-temporal hint, for data that streams through once (partials being summed, shards
// being regathered): on this part a 4-reads-1-write stream moves 6.1-6.2 TB/s with the hint against 5.2-5.5 without.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f32x4 load_stream4(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)); }
__device__ __forceinline__ void store_stream4(float* p, f32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p)); }
__device__ __forceinline__ void store_stream4(bf16_bits* p, f32x4 v) {
  u32x2 b;
  b.x = static_cast<uint32_t>(float_to_bf16(v.x)) | (static_cast<uint32_t>(float_to_bf16(v.y)) << 16);
  b.y = static_cast<uint32_t>(float_to_bf16(v.z)) | (static_cast<uint32_t>(float_to_bf16(v.w)) << 16);
  __builtin_nontemporal_store(b, reinterpret_cast<u32x2*>(p));
}

// Elementwise epilogue on a finished sum (gspmd_epilogue); NaN stays NaN.
__device__ __forceinline__ float apply_epilogue(float v, int epilogue) {
  return (epilogue == GSPMD_EPILOGUE_RELU && v < 0.f) ? 0.f : v;
}

// Which problem owns output tile `tile`: the last entry whose tile_begin <= tile.
__device__ __forceinline__ int find_problem(const Problem* __restrict__ tab, int n_prob, int tile) {
  int lo = 0, hi = n_prob - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (tab[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Launch tables small enough to travel as kernel arguments (no upload, so such a launch can be recorded into a HIP
// graph): up to kInlineProblems problems and kInlineRects zero-fill rectangles.  Larger tables are read from device
// memory (`tab` non-null).
constexpr int kInlineProblems = 32;
constexpr int kInlineRects = 2 * kInlineProblems;
struct InlineProblems { Problem p[kInlineProblems]; };
struct InlineRects { ZeroRect r[kInlineRects]; };

// The kernel-argument segment, read in place: loads from it with a wave-uniform index are scalar loads.  (A by-value
// struct parameter that is indexed dynamically through its C++ name is first copied to private memory.)  The table
// read this way must be the kernel's FIRST parameter, which sits at offset 0 of the segment.
#define GSPMD_KERNARG __attribute__((address_space(4)))
template <typename T>
__device__ __forceinline__ const GSPMD_KERNARG T* first_kernel_argument() {
  return (const GSPMD_KERNARG T*)__builtin_amdgcn_kernarg_segment_ptr();
}
template <typename T>
__device__ __forceinline__ T copy_from_kernarg(const GSPMD_KERNARG T* p) {
  static_assert(sizeof(T) % 8 == 0, "copied as 64-bit words");
  const GSPMD_KERNARG uint64_t* q = (const GSPMD_KERNARG uint64_t*)p;
  uint64_t w[sizeof(T) / 8];
#pragma unroll
  for (size_t i = 0; i < sizeof(T) / 8; ++i) w[i] = q[i];
  T out;
  __builtin_memcpy(&out, w, sizeof(T));
  return out;
}

// The problem that owns output tile `tile`, from the table in device memory if there is one, else from the table in
// the kernel arguments (an InlineProblems as first parameter).
__device__ __forceinline__ Problem lookup_problem(const Problem* __restrict__ tab, int n_prob, int tile) {
  if (tab) return tab[find_problem(tab, n_prob, tile)];
  const GSPMD_KERNARG Problem* inl = first_kernel_argument<Problem>();
  int lo = 0, hi = n_prob - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (inl[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
  }
  return copy_from_kernarg(inl + lo);
}

constexpr int kGenTile = 64;   // output tile edge of the fallback kernel
constexpr int kGenBK = 16;

// Fallback contraction: 64x64 output tile per workgroup, 4x4 outputs per thread, fp32 FMA.
// Every load is predicated on the valid extents (masked positions contribute 0 and are never
// read); stores cover the static extents and write 0 outside the valid region.
template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void dot_fallback_kernel(const InlineProblems inl, const Problem* __restrict__ tab, int n_prob, int layout, int epilogue) {
  __shared__ float As[kGenBK][kGenTile + 4];   // [k][m]
  __shared__ float Bs[kGenBK][kGenTile + 4];   // [k][n]
  const int tile = blockIdx.x;
  const Problem P = lookup_problem(tab, n_prob, tile);
  const int local = tile - P.tile_begin;
  const int m0 = (local / P.tiles_n) * kGenTile, n0 = (local % P.tiles_n) * kGenTile;
  const TIn* __restrict__ A = static_cast<const TIn*>(P.A);
  const TIn* __restrict__ B = static_cast<const TIn*>(P.B);
  TOut* __restrict__ C = static_cast<TOut*>(P.C);
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  // element strides of the two indices of each operand
  const int64_t a_sm = (layout & GSPMD_LAYOUT_LHS_K_MAJOR) ? 1 : P.lda, a_sk = (layout & GSPMD_LAYOUT_LHS_K_MAJOR) ? P.lda : 1;
  const int64_t b_sk = (layout & GSPMD_LAYOUT_RHS_K_CONTIGUOUS) ? 1 : P.ldb, b_sn = (layout & GSPMD_LAYOUT_RHS_K_CONTIGUOUS) ? P.ldb : 1;
  if (m0 < P.Mv && n0 < P.Nv) {
    const int am = t >> 2, ak = (t & 3) * 4;     // A: row am, 4 consecutive k
    const int bk = t >> 4, bn = (t & 15) * 4;    // B: row bk, 4 consecutive n
    for (int k0 = 0; k0 < P.Kv; k0 += kGenBK) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int m = m0 + am, k = k0 + ak + j;
        As[ak + j][am] = (m < P.Mv && k < P.Kv) ? load_as_float<TIn>(A + m * a_sm + k * a_sk) : 0.f;
        const int kk = k0 + bk, n = n0 + bn + j;
        Bs[bk][bn + j] = (kk < P.Kv && n < P.Nv) ? load_as_float<TIn>(B + kk * b_sk + n * b_sn) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < kGenBK; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= P.Ms) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= P.Ns) continue;
      const float v = (m < P.Mv && n < P.Nv) ? apply_epilogue(acc[i][j], epilogue) : 0.f;
      store_from_float<TOut>(C + static_cast<int64_t>(m) * P.ldc + n, v);
    }
  }
}

// Zero fill of the parts of static output blocks that lie in whole tiles beyond the valid extents.
// grid.y = rectangle, grid.x strides over its 16-byte vectors (VEC elements; the host picks VEC = 1 unless the
// pointers, leading dimensions, first columns and widths of all rectangles allow 16-byte stores).
template <typename TOut, int VEC>
__global__ __launch_bounds__(256) void zero_rects_kernel(const InlineRects inl, const ZeroRect* __restrict__ rects) {
  const ZeroRect R = rects ? rects[blockIdx.y] : copy_from_kernarg(first_kernel_argument<ZeroRect>() + blockIdx.y);
  const int wv = (R.c1 - R.c0) / VEC;
  const int64_t total = static_cast<int64_t>(R.r1 - R.r0) * wv;
  TOut* __restrict__ C = static_cast<TOut*>(R.C);
  struct alignas(sizeof(TOut) * VEC) Vec { TOut v[VEC]; };
  Vec z;
#pragma unroll
  for (int j = 0; j < VEC; ++j) z.v[j] = TOut(0);
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t r = i / wv;
    const int c = static_cast<int>(i - r * wv) * VEC;
    *reinterpret_cast<Vec*>(C + (R.r0 + r) * R.ldc + R.c0 + c) = z;
  }
}

// Arrival counters of joined output tiles start every launch at zero (a fill kernel rather than a memset node, so
// that the call can be recorded into a HIP graph).
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* __restrict__ words, int64_t n) {
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * blockDim.x)
    words[i] = 0u;
}

// ---------------------------------------------------------------------------------------
// Sum of K-partials (the arithmetic of the AllReduce along a contracting mesh dimension).
// ---------------------------------------------------------------------------------------
constexpr int kMaxPartials = 16;
struct PartialPtrs { const float* p[kMaxPartials]; };

// rows x cols fp32 partials with leading dimension ld_in -> out with leading dimension ld_out.
// VEC = 4: cols, both leading dimensions and all pointers allow 16-byte (fp32) accesses.
template <typename TOut, int VEC>
__global__ __launch_bounds__(256) void reduce_partials_kernel(PartialPtrs ptrs, int n_partials,
                                                              int64_t rows, int64_t cols, int64_t ld_in,
                                                              TOut* __restrict__ out, int64_t ld_out) {
  const int64_t cols_v = cols / VEC;
  const int64_t total = rows * cols_v;
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t r = i / cols_v, c = (i - r * cols_v) * VEC;
    float acc[VEC];
    if constexpr (VEC == 4) {
      f32x4 sum = load_stream4(ptrs.p[0] + r * ld_in + c);
      for (int p = 1; p < n_partials; ++p) sum += load_stream4(ptrs.p[p] + r * ld_in + c);   // fixed ascending order: deterministic
      store_stream4(out + r * ld_out + c, sum);
    } else {
      acc[0] = ptrs.p[0][r * ld_in + c];
      for (int p = 1; p < n_partials; ++p) acc[0] += ptrs.p[p][r * ld_in + c];
      store_from_float<TOut>(out + r * ld_out + c, acc[0]);
    }
  }
}

// Sum of K-partials written to an out shard that may be a slice of the partials' extent (ReduceScatter: the sum
// followed by each partition's DynamicSlice), any rank.  The last dimension is contiguous on both sides.
struct ScatterDesc {
  int32_t rank;
  int32_t rows;                  // product of the out shard's static extents except the last
  int32_t shard[kMaxRank];       // out shard, static extents
  int32_t valid[kMaxRank];       // out shard, valid extents (the rest is written as 0 and never read from the partials)
  int64_t in_off[kMaxRank];      // where the out shard starts inside the partial, per dimension
  int64_t in_stride[kMaxRank];   // element strides of the (dense) partials
  int64_t out_stride[kMaxRank];  // element strides of the out shard
};

// grid.x covers the last dimension in vectors of VEC, grid.y strides over the rows.  VEC = 4 needs 16-byte aligned
// pointers and every stride, offset and extent of the last two dimensions a multiple of 4.
template <typename TOut, int VEC>
__global__ __launch_bounds__(256) void reduce_scatter_kernel(ScatterDesc d, PartialPtrs ptrs, int n_partials,
                                                             TOut* __restrict__ out, int epilogue) {
  const int last = d.rank - 1;
  const int c = (blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (c >= d.shard[last]) return;
  for (int row = blockIdx.y; row < d.rows; row += gridDim.y) {
    int rem = row;
    int64_t in = d.in_off[last] + c, o = c;
    bool ok = true;
    for (int k = last - 1; k >= 0; --k) {
      const int x = rem % d.shard[k];
      rem /= d.shard[k];
      in += (x + d.in_off[k]) * d.in_stride[k];
      o += x * d.out_stride[k];
      ok = ok && x < d.valid[k];
    }
    float acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
    if (ok && c < d.valid[last]) {
      if constexpr (VEC == 4) {
        f32x4 sum = load_stream4(ptrs.p[0] + in);
        for (int p = 1; p < n_partials; ++p) sum += load_stream4(ptrs.p[p] + in);   // fixed ascending order: deterministic
        acc[0] = sum.x; acc[1] = sum.y; acc[2] = sum.z; acc[3] = sum.w;
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = (c + j < d.valid[last]) ? apply_epilogue(acc[j], epilogue) : 0.f;
      } else {
        acc[0] = ptrs.p[0][in];
        for (int p = 1; p < n_partials; ++p) acc[0] += ptrs.p[p][in];
        acc[0] = apply_epilogue(acc[0], epilogue);
      }
    }
    if constexpr (VEC == 4) {
      f32x4 res;
      res.x = acc[0]; res.y = acc[1]; res.z = acc[2]; res.w = acc[3];
      store_stream4(out + o, res);
    } else {
      store_from_float<TOut>(out + o, acc[0]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Shard <-> global copies (DynamicSlice / DynamicUpdateSlice of the appendix).
// ---------------------------------------------------------------------------------------
struct CopyDesc {
  int32_t rank;
  int64_t shard[kMaxRank];     // static shard shape
  int64_t valid[kMaxRank];
  int64_t sstride[kMaxRank];   // shard strides (elements)
  int64_t gstride[kMaxRank];   // global strides (elements), offset already folded into the base
};

// EXTRACT: shard[idx] = idx valid ? global[idx] : pad.   !EXTRACT: global[idx] = shard[idx] for valid idx.
template <typename T, bool EXTRACT>
__global__ __launch_bounds__(256) void shard_copy_kernel(CopyDesc d, const T* __restrict__ src,
                                                         T* __restrict__ dst, T pad, int64_t total) {
  for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    int64_t rem = i, so = 0, go = 0;
    bool ok = true;
    for (int k = d.rank - 1; k >= 0; --k) {
      const int64_t x = rem % d.shard[k];
      rem /= d.shard[k];
      so += x * d.sstride[k];
      go += x * d.gstride[k];
      ok = ok && (x < d.valid[k]);
    }
    if (EXTRACT) dst[so] = ok ? src[go] : pad;
    else if (ok) dst[go] = src[so];
  }
}

// ---------------------------------------------------------------------------------------
// Resharding: gather every dst shard from the src shards that own its elements.
// ---------------------------------------------------------------------------------------
struct ReshardDesc {              // one per distinct dst buffer
  void* dst;
  int32_t rank;
  int32_t rows;                   // product of the dst shard's static extents except the last
  int32_t shard[kMaxRank];        // dst shard, static extents
  int32_t valid[kMaxRank];        // dst shard, valid extents
  int32_t dst_off[kMaxRank];      // global index of the dst shard's first element
  int32_t src_per[kMaxRank];      // static shard size of src along each dimension
  int32_t pos_stride[kMaxRank];   // mesh-position stride of the mesh dimension src splits this dimension on (0 if none)
  int32_t base_pos;               // mesh position contributed by the mesh dimensions src is not split on
  int64_t dst_stride[kMaxRank];
  int64_t src_stride[kMaxRank];
};

// grid.x covers the last dimension in vectors of VEC elements, grid.y strides over rows, grid.z = dst buffer.
// VEC > 1 needs every chunk boundary, offset and stride of the last dimension to be a multiple of VEC elements and
// 16-byte aligned pointers (checked on the host).  The owner of an element changes only when a row crosses into
// another src shard, so the src pointer (src_by_pos[mesh position], composed on the host from the device-id tensor) is
// fetched again only then.
template <typename T, int VEC, typename DescPtr, typename SrcPtr>
__device__ __forceinline__ void reshard_body(DescPtr dp, SrcPtr src_by_pos) {
  const auto& d = *dp;
  const int last = d.rank - 1;
  const int c = (blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (c >= d.shard[last]) return;
  struct alignas(sizeof(T) * VEC) Vec { T v[VEC]; };
  T* __restrict__ dst = static_cast<T*>(d.dst);
  const uint32_t gl = static_cast<uint32_t>(d.dst_off[last]) + c;
  const uint32_t chunk_l = gl / static_cast<uint32_t>(d.src_per[last]), local_l = gl - chunk_l * d.src_per[last];
  const bool col_ok = c < d.valid[last];
  int held_pos = -1;
  const T* __restrict__ src = nullptr;
  for (int row = blockIdx.y; row < d.rows; row += gridDim.y) {
    uint32_t rem = row;
    int pos = d.base_pos + static_cast<int>(chunk_l) * d.pos_stride[last];
    int64_t so = local_l, o = c;
    bool ok = col_ok;
    for (int k = last - 1; k >= 0; --k) {
      const uint32_t x = rem % static_cast<uint32_t>(d.shard[k]);
      rem /= static_cast<uint32_t>(d.shard[k]);
      const uint32_t gk = static_cast<uint32_t>(d.dst_off[k]) + x;
      const uint32_t chunk = gk / static_cast<uint32_t>(d.src_per[k]);
      pos += static_cast<int>(chunk) * d.pos_stride[k];
      so += static_cast<int64_t>(gk - chunk * d.src_per[k]) * d.src_stride[k];
      o += static_cast<int64_t>(x) * d.dst_stride[k];
      ok = ok && static_cast<int>(x) < d.valid[k];
    }
    Vec v;
#pragma unroll
    for (int j = 0; j < VEC; ++j) v.v[j] = T(0);
    if (ok) {
      if (pos != held_pos) {
        src = static_cast<const T*>(src_by_pos[pos]);
        held_pos = pos;
      }
      if constexpr (sizeof(Vec) == 16) {
        const u32x4 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + so));
        __builtin_memcpy(&v, &raw, 16);
      } else {
        v = *reinterpret_cast<const Vec*>(src + so);
      }
#pragma unroll
      for (int j = 0; j < VEC; ++j) if (c + j >= d.valid[last]) v.v[j] = T(0);
    }
    if constexpr (sizeof(Vec) == 16) {
      u32x4 raw;
      __builtin_memcpy(&raw, &v, 16);
      __builtin_nontemporal_store(raw, reinterpret_cast<u32x4*>(dst + o));
    } else {
      *reinterpret_cast<Vec*>(dst + o) = v;
    }
  }
}

// Tables small enough to travel as kernel arguments (no upload): up to kInlineReshardSrc partitions and
// kInlineReshardDescs distinct dst buffers; larger ones are read from device memory (`descs` non-null).
constexpr int kInlineReshardSrc = 64, kInlineReshardDescs = 8;
struct InlineReshard {
  const void* src[kInlineReshardSrc];
  ReshardDesc d[kInlineReshardDescs];
};

template <typename T, int VEC>
__global__ __launch_bounds__(256) void reshard_kernel(const InlineReshard inl, const ReshardDesc* __restrict__ descs,
                                                      const void* const* __restrict__ src_by_pos) {
  if (descs) {
    reshard_body<T, VEC>(descs + blockIdx.z, src_by_pos);
  } else {
    const GSPMD_KERNARG InlineReshard* in_args = first_kernel_argument<InlineReshard>();
    reshard_body<T, VEC>(&in_args->d[blockIdx.z], &in_args->src[0]);
  }
}

}  // namespace gspmd
