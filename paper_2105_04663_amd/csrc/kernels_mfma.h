// bf16 MFMA contraction for gfx950 (CDNA4): C[m,n] = sum_k A[m,k] * B[k,n], A row-major with k
// contiguous, B row-major with n contiguous ("NN"), fp32 accumulation in the matrix cores.
//
// Workgroup tile 256 x 256, K step 64, 8 wavefronts (2 along m x 4 along n), each owning a
// 128 x 64 block as 4 x 2 MFMA 32x32x16 tiles (128 accumulator registers per lane).
// LDS holds two stages of an A tile [256 m][64 k] and a B tile [64 k][256 n], both in the
// operands' own memory order and filled by direct global->LDS loads (no register staging);
// 16-byte chunks are XOR-swizzled inside a row -- on the global-address side, since a direct
// load writes lane i's 16 bytes at LDS base + 16*i -- so that fragment reads spread over all
// banks.  The B fragment needs k along the lane's registers while memory has n contiguous: it
// is read with the LDS transpose read (ds_read_b64_tr_b16), which hands lane j of a 16-lane
// group column j of a 4 x 16 block.
// The MFMA is issued with the roles of the two operands exchanged (rhs fragment as the first
// operand): the accumulator then holds, per lane, 4 consecutive n of one row m, so the epilogue
// stores 8 (bf16) or 16 (fp32) contiguous bytes per lane.
// The K loop over full tiles is hand-scheduled assembly (mainloop_asm.h, written by
// gen_mainloop.py): the two wave groups ping-pong between an LDS-read phase and an MFMA phase.
//
// Pad + mask (Section 4.1) is fused into the tile loads: rows/columns beyond the valid extents
// are redirected to the last valid row/chunk (their results are never stored) and positions
// beyond the valid K are replaced by zero in BOTH operands (the partial last K tile goes through
// registers); no element at an index >= the valid length of any dimension is ever read.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_basic.h"
#include "mainloop_asm.h"
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

// s_waitcnt immediate for gfx9: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 15) << 8); }
#define GSPMD_WAIT_ALL() __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0))

// 16 bytes per lane from sbase + voff (bytes) straight into LDS at lds_addr + lane*16.  The compiler
// does not see this as an LDS write: every consumer is ordered by an explicit s_waitcnt vmcnt + barrier.
__device__ __forceinline__ void global_to_lds16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}

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
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 2, wn = wave & 3;     // wm is also the ping-pong group

  const int tile = blockIdx.x;
  const Problem P = tab[find_problem(tab, n_prob, tile)];
  const int local = tile - P.tile_begin;
  const int m0 = (local / P.tiles_n) * kMfmaBM, n0 = (local % P.tiles_n) * kMfmaBN;

  float16_t acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const bool live = m0 < P.Mv && n0 < P.Nv && P.Kv > 0;
  if (live) {
    const bf16_bits* __restrict__ Abase = static_cast<const bf16_bits*>(P.A) + static_cast<int64_t>(m0) * P.lda;
    const bf16_bits* __restrict__ Bbase = static_cast<const bf16_bits*>(P.B) + n0;
    const int nk_full = P.Kv / kMfmaBK;
    const int nk = (P.Kv + kMfmaBK - 1) / kMfmaBK;

    // ---- tile loads: 4 A and 4 B wave-instructions of 1 KiB each per wave
    int a_off[4], b_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = (wave * 4 + j) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz_a(r);
      const int rr = min(m0 + r, P.Mv - 1) - m0;               // rows past the valid extent: reuse the last valid row
      a_off[j] = (rr * P.lda + c * 8) * 2;      // bytes
      const int kr = (wave * 4 + j) * 2 + (lane >> 5);
      const int cn = (lane & 31) ^ swz_b(kr);
      int n = n0 + cn * 8;
      if (n >= P.Nv) n = ((P.Nv - 1) >> 3) << 3;               // chunks past the valid extent: reuse the last valid chunk
      b_off[j] = (kr * P.ldb + (n - n0)) * 2;   // bytes
    }
    // last, partial K tile: through registers, zeroing what lies beyond the valid K in BOTH operands
    auto load_tail = [&](int kt, int stage) {
      const int k0 = kt * kMfmaBK;
      const bf16_bits* ab = Abase + k0;
      const bf16_bits* bb = Bbase + static_cast<int64_t>(k0) * P.ldb;
      unsigned char* sa = smem + stage * kStage + wave * 4096 + lane * 16;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = (wave * 4 + j) * 8 + (lane >> 3);
        const int k = k0 + ((lane & 7) ^ swz_a(r)) * 8;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (k < P.Kv) {
          v = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const unsigned char*>(ab) + a_off[j]);
          if (k + 8 > P.Kv) v = mask_tail8(v, P.Kv - k);
        }
        *reinterpret_cast<u32x4_t*>(sa + j * 1024) = v;
        const int kr = k0 + (wave * 4 + j) * 2 + (lane >> 5);
        u32x4_t w = {0u, 0u, 0u, 0u};
        if (kr < P.Kv) w = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const unsigned char*>(bb) + b_off[j]);
        *reinterpret_cast<u32x4_t*>(sa + kStageA + j * 1024) = w;
      }
      GSPMD_WAIT_ALL();
    };
    // one of the 8 wave-instructions of full tile kt (j < 4: A, else B); kt is clamped so that a
    // load issued past the last full tile re-reads a valid tile into a stage nobody reads any more
    auto load_one = [&](int kt, int j) {
      const int kc = min(kt, nk_full - 1);
      const bf16_bits* ab = Abase + kc * kMfmaBK;
      const bf16_bits* bb = Bbase + static_cast<int64_t>(kc) * kMfmaBK * P.ldb;
      const uint32_t sa = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem)) + (kt & 1) * kStage + wave * 4096;
      if (j < 4) global_to_lds16(ab, a_off[j], sa + j * 1024);
      else global_to_lds16(bb, b_off[j - 4], sa + kStageA + (j - 4) * 1024);
    };
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
    // fragment reads and MFMAs of half a K step in compiler-scheduled form (partial last tile only)
    bf16x8_t fa[2][4], fb[2][2];
    auto read_frags = [&](int stage, int hh) {
      const unsigned char* base = smem + stage * kStage;
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) {
        const int kk = hh * 2 + k2;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
          fa[k2][mi] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(base + a_frag[kk] + mi * 32 * 128));
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const unsigned char* p = base + b_frag[ni] + kk * 16 * 512;
          short8_t both;
          both.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p));
          both.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p + 4 * 512));
          fb[k2][ni] = __builtin_bit_cast(bf16x8_t, both);
        }
      }
    };
    auto mma_all = [&]() {
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][ni], fa[kk][mi], acc[mi][ni], 0, 0, 0);
    };

    if (nk_full > 0) {
      // ---- prologue: every wave loads its share of tile 0; group 1 also its share of tile 1
#pragma unroll
      for (int j = 0; j < 8; ++j) load_one(0, j);
      if (wm == 1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) load_one(1, j);
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(8, 0));
      } else {
        GSPMD_WAIT_ALL();
      }
      __builtin_amdgcn_s_barrier();
      {   // ---- K loop over the full tiles: hand-scheduled assembly, see gen_mainloop.py for the register plan
        const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
        const uint32_t ard = lds0 + a_frag[0];
        uint32_t brd0 = lds0 + b_frag[0], brd1 = lds0 + b_frag[1];
        const int first = min(wm == 0 ? 1 : 2, nk_full - 1);
        unsigned long long aptr = reinterpret_cast<unsigned long long>(Abase + first * kMfmaBK);
        unsigned long long bptr = reinterpret_cast<unsigned long long>(Bbase + static_cast<int64_t>(first) * kMfmaBK * P.ldb);
        uint32_t nadv = nk_full - 1 - first;
        uint32_t wr = lds0 + (wm == 0 ? kStage : 0) + wave * 4096;
        uint32_t nkr = nk_full;
        const uint32_t bstep = static_cast<uint32_t>(P.ldb) * (kMfmaBK * 2);
#define GSPMD_MAINLOOP_OPERANDS \
        : "+{v[0:15]}"(acc[0][0]), "+{v[16:31]}"(acc[0][1]), "+{v[32:47]}"(acc[1][0]), "+{v[48:63]}"(acc[1][1]), \
          "+{v[64:79]}"(acc[2][0]), "+{v[80:95]}"(acc[2][1]), "+{v[96:111]}"(acc[3][0]), "+{v[112:127]}"(acc[3][1]), \
          [brd0] "+v"(brd0), [brd1] "+v"(brd1), "+{s[40:41]}"(aptr), "+{s[42:43]}"(bptr), "+{s44}"(wr), "+{s45}"(nkr), "+{s46}"(nadv) \
        : [ard] "v"(ard), [ao0] "v"(a_off[0]), [ao1] "v"(a_off[1]), [ao2] "v"(a_off[2]), [ao3] "v"(a_off[3]), \
          [bo0] "v"(b_off[0]), [bo1] "v"(b_off[1]), [bo2] "v"(b_off[2]), [bo3] "v"(b_off[3]), "{s47}"(bstep) \
        : GSPMD_MAINLOOP_CLOBBERS
        if (wm == 0) {
          asm volatile(GSPMD_MAINLOOP_G0 GSPMD_MAINLOOP_OPERANDS);
        } else {
          asm volatile(GSPMD_MAINLOOP_G1 GSPMD_MAINLOOP_OPERANDS);
        }
      }
      GSPMD_WAIT_ALL();
      __syncthreads();
    }
    if (nk > nk_full) {   // partial last K tile, not pipelined
      load_tail(nk_full, 0);
      __syncthreads();
      read_frags(0, 0);
      mma_all();
      read_frags(0, 1);
      mma_all();
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
