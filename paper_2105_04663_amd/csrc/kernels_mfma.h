// bf16 MFMA contraction for gfx950 (CDNA4): C[m,n] = sum_k A[m,k] * B[k,n], A row-major with k
// contiguous, B row-major with n contiguous ("NN"), fp32 accumulation in the matrix cores.
//
// Workgroup tile 256 x 256, K step 64, 8 wavefronts (2 along m x 4 along n), each owning a
// 128 x 64 block as 4 x 2 MFMA 32x32x16 tiles (128 accumulator registers per lane).
// LDS holds two stages of an A tile [256 m][64 k] and a B tile [64 k][256 n], both in the
// operands' own memory order; 16-byte chunks are XOR-swizzled inside a row so that fragment
// reads spread over all banks.  The B fragment needs k along the lane's registers while memory
// has n contiguous: it is read with the LDS transpose read (ds_read_b64_tr_b16), which hands
// lane j of a 16-lane group column j of a 4 x 16 block.
// The MFMA is issued with the roles of the two operands exchanged (rhs fragment as the first
// operand): the accumulator then holds, per lane, 4 consecutive n of one row m, so the epilogue
// stores 8 (bf16) or 16 (fp32) contiguous bytes per lane.
//
// Pad + mask (Section 4.1) is fused into the tile loads: rows/columns beyond the valid extents
// are redirected to the last valid row/chunk (their results are never stored) and positions
// beyond the valid K are replaced by zero in BOTH operands; no element at an index >= the
// valid length of any dimension is ever read.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_basic.h"
#include "plan.h"

namespace gspmd {

constexpr int kMfmaBM = 256, kMfmaBN = 256, kMfmaBK = 64;
constexpr int kMfmaThreads = 512;
constexpr int kStageA = kMfmaBM * kMfmaBK * 2;     // 32 KiB
constexpr int kStageB = kMfmaBK * kMfmaBN * 2;     // 32 KiB
constexpr int kStage = kStageA + kStageB;
constexpr int kMfmaLds = 2 * kStage;               // 128 KiB of the CU's 160 KiB

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(8))) short short8_t;
typedef __attribute__((ext_vector_type(16))) float float16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((address_space(3))) short4_t lds_short4_t;

__device__ __forceinline__ int swz_a(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz_b(int krow) { return ((krow & 3) << 2) ^ (((krow >> 3) & 1) << 1); }

__device__ __forceinline__ u32x4_t mask_tail8(u32x4_t v, int keep) {   // keep first `keep` of 8 bf16
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t m = (2 * d + 1 < keep) ? 0xffffffffu : ((2 * d < keep) ? 0x0000ffffu : 0u);
    v[d] &= m;
  }
  return v;
}

template <typename TOut>
__global__ __launch_bounds__(kMfmaThreads) void dot_mfma_kernel(const Problem* __restrict__ tab, int n_prob) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  const int tile = blockIdx.x;
  const Problem P = tab[find_problem(tab, n_prob, tile)];
  const int local = tile - P.tile_begin;
  const int m0 = (local / P.tiles_n) * kMfmaBM, n0 = (local % P.tiles_n) * kMfmaBN;
  const bf16_bits* __restrict__ Ag = static_cast<const bf16_bits*>(P.A);
  const bf16_bits* __restrict__ Bg = static_cast<const bf16_bits*>(P.B);

  float16_t acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const bool live = m0 < P.Mv && n0 < P.Nv && P.Kv > 0;
  if (live) {
    // ---- global -> register -> LDS staging: 4 A chunks and 4 B chunks of 16 bytes per thread
    const bf16_bits* a_ptr[4];
    const bf16_bits* b_ptr[4];
    int a_lds[4], b_lds[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (t >> 3) + 64 * i, c = t & 7;
      const int grow = min(m0 + row, P.Mv - 1);             // rows past the valid extent: reuse the last valid row
      a_ptr[i] = Ag + static_cast<int64_t>(grow) * P.lda + c * 8;
      a_lds[i] = row * 128 + ((c ^ swz_a(row)) << 4);
      const int krow = (t >> 5) + 16 * i, cn = t & 31;
      int n = n0 + cn * 8;
      if (n >= P.Nv) n = ((P.Nv - 1) >> 3) << 3;            // chunks past the valid extent: reuse the last valid chunk
      b_ptr[i] = Bg + static_cast<int64_t>(krow) * P.ldb + n;
      b_lds[i] = kStageA + krow * 512 + ((cn ^ swz_b(krow)) << 4);
    }
    // ---- fragment read offsets
    int a_frag[4];   // per kk; + mi*32*128 added as an immediate
    {
      const int row = wm * 128 + (lane & 31);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) a_frag[kk] = row * 128 + (((kk * 2 + (lane >> 5)) ^ swz_a(row)) << 4);
    }
    int b_frag[2];   // per ni; + (kk*16 + rd*4)*512 added as an immediate
    {
      const int g = lane >> 4, i = lane & 15;
      const int krow = (g >> 1) * 8 + (i >> 2);
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int nl = wn * 64 + ni * 32 + (g & 1) * 16 + (i & 3) * 4;
        b_frag[ni] = kStageA + krow * 512 + ((((nl >> 3)) ^ swz_b(krow)) << 4) + (nl & 7) * 2;
      }
    }

    const int nk = (P.Kv + kMfmaBK - 1) / kMfmaBK;
    u32x4_t ra[4], rb[4];

    auto load_tile = [&](int kt) {
      const int k0 = kt * kMfmaBK;
      if (k0 + kMfmaBK <= P.Kv) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          ra[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + k0);
          rb[i] = *reinterpret_cast<const u32x4_t*>(b_ptr[i] + static_cast<int64_t>(k0) * P.ldb);
        }
      } else {   // last, partial K tile: zero what lies beyond the valid K in both operands
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int k = k0 + (t & 7) * 8;
          u32x4_t v = {0u, 0u, 0u, 0u};
          if (k < P.Kv) {
            v = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + k0);
            if (k + 8 > P.Kv) v = mask_tail8(v, P.Kv - k);
          }
          ra[i] = v;
          const int kr = k0 + (t >> 5) + 16 * i;
          u32x4_t w = {0u, 0u, 0u, 0u};
          if (kr < P.Kv) w = *reinterpret_cast<const u32x4_t*>(b_ptr[i] + static_cast<int64_t>(k0) * P.ldb);
          rb[i] = w;
        }
      }
    };
    auto store_tile = [&](int stage) {
      unsigned char* base = smem + stage * kStage;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4_t*>(base + a_lds[i]) = ra[i];
        *reinterpret_cast<u32x4_t*>(base + b_lds[i]) = rb[i];
      }
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const bool more = kt + 1 < nk;
      if (more) load_tile(kt + 1);
      const unsigned char* base = smem + (kt & 1) * kStage;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8_t fa[4], fb[2];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
          fa[mi] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(base + a_frag[kk] + mi * 32 * 128));
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const unsigned char* p = base + b_frag[ni] + kk * 16 * 512;
          const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p));
          const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p + 4 * 512));
          short8_t both;
          both.lo = lo; both.hi = hi;
          fb[ni] = __builtin_bit_cast(bf16x8_t, both);
        }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], acc[mi][ni], 0, 0, 0);
      }
      if (more) store_tile((kt + 1) & 1);
      __syncthreads();
    }
  }

  // ---- epilogue: lane holds, for row m, columns n .. n+3 of each 8-column group
  TOut* __restrict__ Cg = static_cast<TOut*>(P.C);
  const bool vec_ok = ((P.ldc & 3) == 0) && ((reinterpret_cast<uintptr_t>(Cg) & 15) == 0);
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int m = m0 + wm * 128 + mi * 32 + (lane & 31);
    if (m >= P.Ms) continue;
    const bool mrow = m < P.Mv;
    TOut* crow = Cg + static_cast<int64_t>(m) * P.ldc;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * 64 + ni * 32 + q * 8 + (lane >> 5) * 4;
        if (n >= P.Ns) continue;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (mrow && n + j < P.Nv) ? acc[mi][ni][q * 4 + j] : 0.f;
        if (vec_ok && n + 4 <= P.Ns) {
          if constexpr (sizeof(TOut) == 4) {
            *reinterpret_cast<float4*>(crow + n) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            ushort4 o;
            o.x = float_to_bf16(v[0]); o.y = float_to_bf16(v[1]); o.z = float_to_bf16(v[2]); o.w = float_to_bf16(v[3]);
            *reinterpret_cast<ushort4*>(crow + n) = o;
          }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (n + j < P.Ns) store_from_float<TOut>(crow + n + j, v[j]);
        }
      }
    }
  }
}

// Launch over `tiles` output tiles; out_dtype selects the store type.  false on a HIP error.
inline bool launch_dot_mfma(const Problem* tab, int n_prob, int tiles, int32_t out_dtype, hipStream_t stream) {
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&dot_mfma_kernel<float>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLds) != hipSuccess) return false;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&dot_mfma_kernel<bf16_bits>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLds) != hipSuccess) return false;
    attr_done = true;
  }
  const dim3 grid(static_cast<unsigned>(tiles)), block(kMfmaThreads);
  if (out_dtype == GSPMD_F32)
    hipLaunchKernelGGL((dot_mfma_kernel<float>), grid, block, kMfmaLds, stream, tab, n_prob);
  else
    hipLaunchKernelGGL((dot_mfma_kernel<bf16_bits>), grid, block, kMfmaLds, stream, tab, n_prob);
  return hipGetLastError() == hipSuccess;
}

}  // namespace gspmd
