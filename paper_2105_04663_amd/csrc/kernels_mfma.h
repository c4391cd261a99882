// bf16 MFMA contraction for gfx950 (CDNA4): C[m,n] = sum_k A[m,k] * B[k,n], fp32 accumulation in the matrix
// cores.  Each operand is either K-contiguous (rows of k) or K-major (rows of m resp. n); the forward einsums have
// A K-contiguous and B K-major ("NN", described below), a weight gradient has both K-major, an input gradient both
// K-contiguous.  The kernel is instantiated per combination (template parameter LAYOUT, GSPMD_LAYOUT_* bits): a
// K-major A uses B's tile format and transpose reads, a K-contiguous B uses A's.
//
// Workgroup tile 256 x 256, 8 wavefronts (2 along m x 4 along n), each owning a 128 x 64 block as 8 x 4
// v_mfma_f32_16x16x32_bf16 tiles (128 accumulator registers per lane), one workgroup per CU.
// LDS (all 160 KiB) holds five stages of a 32-wide K tile, an A part and a B part of 16 KiB each, both in
// the operands' own memory order and filled by direct global->LDS loads (no register staging, no ds_write):
// the B part is [32 k][256 n]; the A parts of the two tiles of a 64-wide K step hold rows 0-127 and rows 128-255 of
// the tile as [128 m][64 k], so that every row is a whole 128-byte line of global memory.
// 16-byte chunks are XOR-swizzled inside a row -- on the global-address side, since a direct load writes lane i's
// 16 bytes at LDS base + 16*i -- so that fragment reads are bank-conflict free.  The B fragment needs k along the
// lane's registers while memory has n contiguous: it is read with the LDS transpose read (ds_read_b64_tr_b16),
// which hands lane j of a 16-lane group column j of a 4 x 16 block.
// The MFMA is issued with the roles of the two operands exchanged (rhs fragment as the first operand): the
// accumulator then holds, per lane, 4 consecutive n of one row m, so the epilogue stores 8 (bf16) or 16 (fp32)
// contiguous bytes per lane.
// The K loop over full 64-wide steps is hand-scheduled assembly (mainloop_asm.h, written by gen_mainloop.py, which
// also documents the schedule): the two wave groups ping-pong between an LDS-read phase and an MFMA phase.
//
// Pad + mask (Section 4.1) is fused into the tile loads: rows/columns beyond the valid extents are redirected to the
// last valid row/chunk (their results are never stored) and positions beyond the valid K are replaced by zero in
// BOTH operands (what is left of K after the full 64-wide steps goes through registers); no element at an index >=
// the valid length of any dimension is ever read.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "kernels_basic.h"
#include "mainloop_asm.h"
#include "plan.h"
#include "tile_index.h"

namespace gspmd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(8))) short short8_t;
typedef __attribute__((ext_vector_type(16))) float float16_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((address_space(3))) short4_t lds_short4_t;

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

// 16 bytes from an address that is only 4-byte aligned
typedef uint32_t u32x4_align4_t __attribute__((ext_vector_type(4), aligned(4)));
typedef __attribute__((address_space(1))) u32x4_t global_u32x4_t;

// Profiling aid (gspmd_set_tile_timeline): one record of eight 64-bit words per workgroup, written by its thread 0.
// Words 0-7 hold the 100 MHz constant-rate counter at: kernel entry (bits 52-63: XCD id << 8 | compute-unit bits
// 8-15 of the hardware id register), tile decoded, first tile loads issued, first tiles landed (K loop starts), K
// loop left, epilogue starts (leftover K and joined sums done), stores issued, stores complete.  `rec` is null
// when the timeline is off; the branch is uniform and costs two scalar instructions per stamp.
constexpr int kTimelineWords = 8;
__device__ __forceinline__ void timeline_stamp(unsigned long long* rec, int word, int t, unsigned long long tag = 0) {
  if (rec == nullptr) return;
  unsigned long long now;
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(now) :: "memory");
  if (t == 0) rec[word] = now | (tag << 52);
}

// Zeros over rows [row_begin, row_end) x columns [col_begin, col_end) of an output block, by all kMfmaThreads threads of
// the workgroup: the rows of the static block below the last tile row's footprint.  `vec`: 16-byte stores are
// aligned (checked by the caller for the block's pointer, row stride and col_begin) and the width is a multiple of them.
template <typename TOut>
__device__ __forceinline__ void zero_rows_below(TOut* __restrict__ C, int ldc, int row_begin, int row_end, int col_begin, int col_end,
                                                bool vec, int t) {
  const int width = col_end - col_begin;
  if (row_end <= row_begin || width <= 0) return;
  if (vec) {
    constexpr int kPer = 16 / static_cast<int>(sizeof(TOut));          // elements per store
    const int per_row = width / kPer;                                  // stores per row
    const int total = (row_end - row_begin) * per_row;
    const u32x4_t z = {0u, 0u, 0u, 0u};
    for (int i = t; i < total; i += kMfmaThreads) {
      const int r = i / per_row, c = (i - r * per_row) * kPer;
      __builtin_nontemporal_store(z, (global_u32x4_t*)(C + static_cast<int64_t>(row_begin + r) * ldc + col_begin + c));
    }
  } else {
    const int total = (row_end - row_begin) * width;
    for (int i = t; i < total; i += kMfmaThreads) {
      const int r = i / width, c = i - r * width;
      store_from_float<TOut>(C + static_cast<int64_t>(row_begin + r) * ldc + col_begin + c, 0.f);
    }
  }
}

// STAGED: the variant for operands whose rows are only 4-byte aligned (an even row stride that is not a multiple of
// 8 elements, e.g. dense shards of 1250 columns): direct global->LDS loads need 16-byte aligned chunks, so every K
// tile goes through registers instead -- the path the other variant uses for what is left of K after its assembly
// loop -- with the next K step's chunks in flight while the current one is multiplied.  Chunks that are only partly
// valid are loaded 4 bytes at a time, so that no read leaves the rows' valid part by more than one element.
template <typename TOut, int LAYOUT, bool STAGED>
__global__ __launch_bounds__(kMfmaThreads) void dot_mfma_kernel(const InlineProblems inl, const Problem* __restrict__ tab, int n_prob, int epilogue,
                                                                float* __restrict__ join_partials, uint32_t* __restrict__ join_counters,
                                                                unsigned long long* __restrict__ timeline, int timeline_records) {
  constexpr bool AKM = (LAYOUT & GSPMD_LAYOUT_LHS_K_MAJOR) != 0, BKC = (LAYOUT & GSPMD_LAYOUT_RHS_K_CONTIGUOUS) != 0;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 2, wn = wave & 3;     // wm is also the ping-pong group

  unsigned long long* const rec = (timeline != nullptr && static_cast<int>(blockIdx.x) < timeline_records)
                                      ? timeline + static_cast<size_t>(blockIdx.x) * kTimelineWords : nullptr;
  if (rec != nullptr) {
    const unsigned where = ((__builtin_amdgcn_s_getreg((31 << 11) | 20) & 15u) << 8) | ((__builtin_amdgcn_s_getreg((31 << 11) | 4) >> 8) & 255u);
    timeline_stamp(rec, 0, t, where);
  }
  const int tile = logical_tile(blockIdx.x, gridDim.x);
  const Problem P = lookup_problem(tab, n_prob, tile);
  const int local = tile - P.tile_begin;            // which of its problem's output tiles this workgroup computes
  int tile_row, n0;
  tile_origin(local, P.Mv, P.tiles_n, &tile_row, &n0);
  // rows [m0, m_end) are this tile's own (valid rows are split evenly over the tile rows, in 16-row blocks); the last
  // tile row also writes the zeros that follow the valid rows, up to the end of its 256-row footprint
  const TileRows own = tile_rows(tile_row, P.Mv);
  const int m0 = own.first, m_end = own.first + own.rows;
  const int m_write_end = m_end == P.Mv ? min(P.Ms, m0 + kMfmaBM) : m_end;

  // acc[bm] holds the four 16x16 tiles (bn = 0..3) of 16-row block bm: element 4*bn + r
  float16_t acc[8];
#pragma unroll
  for (int bm = 0; bm < 8; ++bm)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[bm][r] = 0.f;

  const bool live = m0 < P.Mv && n0 < P.Nv && P.Kv > 0;
  if (live) {
    // the tile's operand panels and the distance (elements) between consecutive 32-wide K tiles
    const bf16_bits* __restrict__ Abase = static_cast<const bf16_bits*>(P.A) + (AKM ? static_cast<int64_t>(m0) : static_cast<int64_t>(m0) * P.lda);
    const bf16_bits* __restrict__ Bbase = static_cast<const bf16_bits*>(P.B) + (BKC ? static_cast<int64_t>(n0) * P.ldb : static_cast<int64_t>(n0));
    const int64_t a_tile = AKM ? static_cast<int64_t>(kMfmaBK) * P.lda : kMfmaBK;
    const int64_t b_tile = BKC ? kMfmaBK : static_cast<int64_t>(kMfmaBK) * P.ldb;
    const int nk64 = P.Kv / (2 * kMfmaBK);    // full 64-wide K steps (the assembly loop)
    const int nkt = 2 * nk64;                 // 32-wide tiles the assembly loop consumes

    // ---- tile loads.  A tile (32 KiB) is 32 wave-instructions of 1 KiB (16 per operand); the four waves of ONE
    // group load a whole tile, wave wn taking instructions 4*wn .. 4*wn+3 of each operand.
    // Group wm loads the tiles of its own parity, hence the half wm of a K-contiguous operand.
    int a_off[4], b_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a_off[j] = AKM ? km_load_offset(wn * 4 + j, lane, m0, m_end, P.lda) : kc_half_load_offset(wn * 4 + j, lane, wm, m0, m_end, P.lda);
      b_off[j] = BKC ? kc_half_load_offset(wn * 4 + j, lane, wm, n0, P.Nv, P.ldb) : km_load_offset(wn * 4 + j, lane, n0, P.Nv, P.ldb);
    }
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
    // address of what tile kt's part holds: k = 32 kt for a K-major operand, the K step's first k for a K-contiguous one
    auto a_tile_ptr = [&](int kt) { return AKM ? Abase + kt * a_tile : Abase + (kt >> 1) * (2 * kMfmaBK); };
    auto b_tile_ptr = [&](int kt) { return BKC ? Bbase + (kt >> 1) * (2 * kMfmaBK) : Bbase + kt * b_tile; };
    // this wave's 8 instructions of tile kt of the main loop; kt is clamped so that a load issued past the loop's
    // last tile re-reads valid memory into a stage nobody reads any more
    auto load_tile = [&](int kt) {
      const int kc = min(kt, nkt - 1);
      const bf16_bits* ab = a_tile_ptr(kc);
      const bf16_bits* bb = b_tile_ptr(kc);
      const uint32_t sa = lds0 + (kt % kNumStages) * kStage + wn * 4096;
#pragma unroll
      for (int j = 0; j < 4; ++j) global_to_lds16(ab, a_off[j], sa + j * 1024);
#pragma unroll
      for (int j = 0; j < 4; ++j) global_to_lds16(bb, b_off[j], sa + kStageA + j * 1024);
    };
    // one 16-byte chunk of a K tile that may be partial: into a register, zero where it lies beyond the valid K (in
    // BOTH operands: the padding may hold anything).  `cols_valid`: valid columns of a K-major operand, counted like
    // `c0`, the tile's first column.
    auto tail_chunk = [&](bool kmajor, const bf16_bits* base, int off, int q, int k0, int c0, int cols_valid) -> u32x4_t {
      u32x4_t v = {0u, 0u, 0u, 0u};
      // operands live in global memory: loads through a global (not generic) pointer count in vmcnt only, so waiting for
      // LDS reads does not wait for them
      typedef __attribute__((address_space(1))) const unsigned char* gptr_t;
      gptr_t at = (gptr_t)(reinterpret_cast<const unsigned char*>(base) + off);
      if (kmajor) {         // a whole k row per 32 lanes
        const int kr = k0 + q * 2 + (lane >> 5);
        if (kr < P.Kv) {
          if constexpr (!STAGED) {
            v = *(__attribute__((address_space(1))) const u32x4_t*)at;
          } else {
            int n = c0 + (((lane & 31) ^ swz_b(q * 2 + (lane >> 5))) << 3);    // the chunk km_load_offset addresses
            if (n >= cols_valid) n = ((cols_valid - 1) >> 3) << 3;
            if (n + 8 <= cols_valid) {
              v = *(__attribute__((address_space(1))) const u32x4_align4_t*)at;
            } else {
#pragma unroll
              for (int d = 0; d < 4; ++d)
                if (n + 2 * d < cols_valid) v[d] = *(__attribute__((address_space(1))) const uint32_t*)(at + 4 * d);
            }
          }
        }
      } else {              // 8 consecutive k per lane
        const int r = q * 16 + (lane >> 2);
        const int k = k0 + ((lane & 3) ^ swz_a(r)) * 8;
        if (k < P.Kv) {
          if constexpr (!STAGED) {
            v = *(__attribute__((address_space(1))) const u32x4_t*)at;
          } else if (k + 8 <= P.Kv) {
            v = *(__attribute__((address_space(1))) const u32x4_align4_t*)at;
          } else {
#pragma unroll
            for (int d = 0; d < 4; ++d)
              if (k + 2 * d < P.Kv) v[d] = *(__attribute__((address_space(1))) const uint32_t*)(at + 4 * d);
          }
          if (k + 8 > P.Kv) v = mask_tail8(v, P.Kv - k);
        }
      }
      return v;
    };
    // this wave's 4 + 4 chunks of tile kt (the four waves of one group bring a whole tile): global memory -> registers,
    // then registers -> the [256][32] / [32][256] parts of a stage
    auto fetch_tail = [&](int kt, u32x4_t (&ta)[4], u32x4_t (&tb)[4]) {
      const int k0 = kt * kMfmaBK;
      const bf16_bits* ab = Abase + kt * a_tile;
      const bf16_bits* bb = Bbase + kt * b_tile;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int q = wn * 4 + j;
        const int ao = AKM ? km_load_offset(q, lane, m0, m_end, P.lda) : kc_load_offset(q, lane, m0, m_end, P.lda);
        const int bo = BKC ? kc_load_offset(q, lane, n0, P.Nv, P.ldb) : km_load_offset(q, lane, n0, P.Nv, P.ldb);
        ta[j] = tail_chunk(AKM, ab, ao, q, k0, m0, m_end);
        tb[j] = tail_chunk(!BKC, bb, bo, q, k0, n0, P.Nv);
      }
    };
    auto store_tail = [&](int stage, const u32x4_t (&ta)[4], const u32x4_t (&tb)[4]) {
      unsigned char* sa = smem + stage * kStage + wn * 4096 + lane * 16;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        *reinterpret_cast<u32x4_t*>(sa + j * 1024) = ta[j];
        *reinterpret_cast<u32x4_t*>(sa + kStageA + j * 1024) = tb[j];
      }
    };
    // ---- fragment read offsets inside a stage, for the tail's [256][32] / [32][256] parts
    const int a_frag = AKM ? km_frag_offset(wm * 128, lane) : kc_frag_offset(wm * 128, lane);
    const int b_frag = kStageA + (BKC ? kc_frag_offset(wn * 64, lane) : km_frag_offset(wn * 64, lane));
    // fragment reads and MFMAs of one K tile in compiler-scheduled form (what is left of K after the assembly loop)
    bf16x8_t fa[8], fb[4];
    auto read_kc = [&](const unsigned char* p) {
      return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(p));
    };
    auto read_km = [&](const unsigned char* p) {
      short8_t both;
      both.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p));
      both.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_t*)(p + 4 * 512));
      return __builtin_bit_cast(bf16x8_t, both);
    };
    auto read_frags = [&](int stage) {
      const unsigned char* base = smem + stage * kStage;
#pragma unroll
      for (int bm = 0; bm < 8; ++bm) fa[bm] = AKM ? read_km(base + (a_frag ^ (bm << 5))) : read_kc(base + a_frag + bm * 1024);
#pragma unroll
      for (int bn = 0; bn < 4; ++bn) fb[bn] = BKC ? read_kc(base + b_frag + bn * 1024) : read_km(base + (b_frag ^ (bn << 5)));
    };
    auto mma_all = [&]() {
#pragma unroll
      for (int bm = 0; bm < 8; ++bm)
#pragma unroll
        for (int bn = 0; bn < 4; ++bn) {
          float4_t c = {acc[bm][4 * bn], acc[bm][4 * bn + 1], acc[bm][4 * bn + 2], acc[bm][4 * bn + 3]};
          c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[bn], fa[bm], c, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[bm][4 * bn + r] = c[r];
        }
    };

    if constexpr (STAGED) {
      // ---- every K tile through registers, two tiles (one per wave group) per step; the next step's chunks are in
      // flight while this step is multiplied
      const int ntiles = (P.Kv + kMfmaBK - 1) / kMfmaBK;
      u32x4_t ta[4], tb[4];
      if (wm < ntiles) fetch_tail(wm, ta, tb);
      for (int kt = 0; kt < ntiles; kt += 2) {
        const int here = min(2, ntiles - kt);
        if (wm < here) store_tail(wm, ta, tb);
        __syncthreads();
        if (kt + 2 + wm < ntiles) fetch_tail(kt + 2 + wm, ta, tb);
        read_frags(0);
        mma_all();
        if (here > 1) {
          read_frags(1);
          mma_all();
        }
        __syncthreads();
      }
    } else {
    timeline_stamp(rec, 1, t);
    if (nk64 > 0) {
      // ---- prologue: group 0 loads tiles 0 and 2, group 1 tiles 1 and 3; tiles 0 and 1 must have landed
      load_tile(wm);
      load_tile(wm + 2);
      timeline_stamp(rec, 2, t);
      __builtin_amdgcn_s_waitcnt(waitcnt_imm(8, 0));
      __builtin_amdgcn_s_barrier();
      timeline_stamp(rec, 3, t);
      {   // ---- K loop over the full 64-wide steps: hand-scheduled assembly, see gen_mainloop.py for the register plan
        // a K-contiguous operand is read from the part that holds this wave's rows: half wm of the lhs, wn >> 1 of the rhs
        const uint32_t ard = lds0 + (AKM ? a_frag : kc_half_frag_offset(0, lane));
        const uint32_t brd = lds0 + (BKC ? kStageA + kc_half_frag_offset((wn & 1) * 64, lane) : b_frag);
        uint32_t astage = wm * kStage, bstage = (wn >> 1) * kStage;
        const int first = min(4 + wm, nkt - 1);           // group 0 goes on with tiles 4, 6, ..; group 1 with 5, 7, ..
        unsigned long long aptr = reinterpret_cast<unsigned long long>(a_tile_ptr(first));
        unsigned long long bptr = reinterpret_cast<unsigned long long>(b_tile_ptr(first));
        uint32_t nadv = (nkt - 1 - first) / 2;
        const uint32_t wrbase = lds0 + wn * 4096;
        uint32_t wstage = ((4 + wm) % kNumStages) * kStage, rstage = 0;
        uint32_t nkr = nk64;
        // 16-row blocks of each group's half (rows 0-127 / 128-255 of the tile) that hold rows of this tile: the loop
        // variant for fewer than 8 skips the reads and MFMAs of the others (their results would never be stored).
        // Group 1 has variants for 4 to 8 blocks; group 0 for 4, 6 and 8 (a tile that ends inside its half belongs to
        // a problem of at most 128 rows; group 1 then runs its shortest variant for nothing but its loads).
        const int g1_rows = own.rows - 128;
        const int g1_blocks = g1_rows <= 64 ? 4 : (g1_rows + 15) >> 4;
        const int g0_blocks = own.rows <= 64 ? 4 : (own.rows <= 96 ? 6 : 8);
        const uint32_t astep = static_cast<uint32_t>(a_tile) * 4, bstep = static_cast<uint32_t>(b_tile) * 4;   // one K step, bytes
#define GSPMD_MAINLOOP_OPERANDS \
        : "+{v[0:15]}"(acc[0]), "+{v[16:31]}"(acc[1]), "+{v[32:47]}"(acc[2]), "+{v[48:63]}"(acc[3]), \
          "+{v[64:79]}"(acc[4]), "+{v[80:95]}"(acc[5]), "+{v[96:111]}"(acc[6]), "+{v[112:127]}"(acc[7]), \
          "+{s[40:41]}"(aptr), "+{s[42:43]}"(bptr), "+{s45}"(nkr), "+{s46}"(nadv), "+{s52}"(wstage), "+{s53}"(rstage), \
          "+{s55}"(astage), "+{s56}"(bstage) \
        : [ard] "v"(ard), [brd] "v"(brd), [ao0] "v"(a_off[0]), [ao1] "v"(a_off[1]), [ao2] "v"(a_off[2]), [ao3] "v"(a_off[3]), \
          [bo0] "v"(b_off[0]), [bo1] "v"(b_off[1]), [bo2] "v"(b_off[2]), [bo3] "v"(b_off[3]), "{s44}"(wrbase), "{s47}"(bstep), "{s54}"(astep) \
        : GSPMD_MAINLOOP_CLOBBERS
        // the four waves of a group issue their tile loads after different MFMAs, so that the CU's
        // texture-address unit sees one load at a time
#define GSPMD_RUN_WAVES(NAME) \
          switch (wn) { \
            case 0: asm volatile(NAME##_W0 GSPMD_MAINLOOP_OPERANDS); break; \
            case 1: asm volatile(NAME##_W1 GSPMD_MAINLOOP_OPERANDS); break; \
            case 2: asm volatile(NAME##_W2 GSPMD_MAINLOOP_OPERANDS); break; \
            default: asm volatile(NAME##_W3 GSPMD_MAINLOOP_OPERANDS); break; \
          }
#define GSPMD_RUN_MAINLOOP(L) \
        if (wm == 0) { \
          if (g0_blocks == 8) { GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G0) } \
          else if (g0_blocks == 6) { GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G0R6) } \
          else { GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G0R4) } \
        } else { \
          switch (g1_blocks) { \
            case 8: GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G1) break; \
            case 7: GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G1R7) break; \
            case 6: GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G1R6) break; \
            case 5: GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G1R5) break; \
            default: GSPMD_RUN_WAVES(GSPMD_MAINLOOP_L##L##_G1R4) break; \
          } \
        }
        if constexpr (LAYOUT == 0) { GSPMD_RUN_MAINLOOP(0) }
        else if constexpr (LAYOUT == 1) { GSPMD_RUN_MAINLOOP(1) }
        else if constexpr (LAYOUT == 2) { GSPMD_RUN_MAINLOOP(2) }
        else { GSPMD_RUN_MAINLOOP(3) }
      }
    }
    // ---- what is left of K (< 64): up to two tiles, the last one possibly partial.  Group 0 fetches the first and
    // group 1 the second as soon as they leave the loop (group 0 a phase earlier), both in flight together; they go
    // through registers (zeroed beyond the valid K) into stages 0 and 1 once every load of the loop has landed.
    timeline_stamp(rec, 4, t);
    const int ntail = (P.Kv - nkt * kMfmaBK + kMfmaBK - 1) / kMfmaBK;
    {
      u32x4_t ta[4], tb[4];
      if (wm < ntail) fetch_tail(nkt + wm, ta, tb);
      // Without leftover tiles nothing follows the loop but the epilogue, and that needs no barrier: the loop ends with
      // no tile load in flight, and every wave's last LDS read was complete before the last barrier that both groups
      // passed, so a wave may overwrite LDS (its epilogue's staging slice) as soon as its own MFMAs are done -- group 0
      // a phase before group 1.
      if (nk64 > 0 && ntail > 0) {
        GSPMD_WAIT_ALL();
        __syncthreads();
      }
      if (ntail > 0) {
        if (wm < ntail) store_tail(wm, ta, tb);
        __syncthreads();
        read_frags(0);
        mma_all();
        if (ntail > 1) {
          read_frags(1);
          mma_all();
        }
        __syncthreads();
      }
    }
    }   // !STAGED
  }

  // ---- joined problems (a contracting dimension split over partitions, Section 4.2, or one K range cut in pieces):
  // every contribution to an output tile is written to its slot of the workspace as fp32, in the accumulators' own
  // lane order (each wave-instruction stores 1 KiB of consecutive addresses); the workgroup that arrives last at the
  // tile's counter adds the slots in ascending order -- a fixed order of fp32 additions, whoever arrives last -- and
  // goes on to the epilogue with the sum.  No workgroup waits for another.
  // Compute units of different XCDs do not share an L2, so the slots are written and read with device-scope accesses
  // (the sc1 cache policy: stores go through to memory, loads do not take a stale line), ordered around the device-
  // scope counter update by a wait for the stores and the workgroup barriers.  A release fence would do the same for
  // plain stores, but it writes back the XCD's whole L2 and was measured to cost tens of microseconds per tile; an
  // acquire fence would drop every operand panel the XCD has cached.
  if (P.join_count > 1) {
    constexpr int kDeviceScope = 16 | 2;                   // sc1, and nt: a slot is written once and read once (measured +1 to 2 %)
    const int S = P.join_count;
    const int64_t jt = static_cast<int64_t>(P.join_first) + local;
    const __amdgpu_buffer_rsrc_t slots = __builtin_amdgcn_make_buffer_rsrc(join_partials + ((jt * S) << 16), 0, S << 18, 0x00020000);
    const int at = (wave * 2048 + lane) * 16;              // this lane's place inside a slot; quad q at + q KiB
#pragma unroll
    for (int bm = 0; bm < 8; ++bm)
#pragma unroll
      for (int bn = 0; bn < 4; ++bn) {
        const float4_t v = {acc[bm][4 * bn], acc[bm][4 * bn + 1], acc[bm][4 * bn + 2], acc[bm][4 * bn + 3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), slots, at, (P.join_slot << 18) + (bm * 4 + bn) * 1024, kDeviceScope);
      }
    GSPMD_WAIT_ALL();                                      // this wave's stores have reached memory
    __syncthreads();                                       // ... and so have the other seven waves'
    uint32_t* flag = reinterpret_cast<uint32_t*>(smem);
    if (t == 0) *flag = __hip_atomic_fetch_add(join_counters + jt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t before = *flag;
    if (before != static_cast<uint32_t>(S - 1)) {
      if (rec != nullptr && t == 0) rec[5] = rec[6] = rec[7] = 0;      // not this launch's last arriver at the tile
      return;
    }
    // The sum over the slots in ascending order.  This workgroup's own contribution is still in its accumulators, so
    // only the other S - 1 slots are read back: a quarter of the accumulators (8 quads) at a time, up to three slots
    // (96 spare registers) in flight together -- one round trip to memory per quarter for up to four contributions.
    // Until the own slot's turn comes, the sum of the slots before it is kept in the registers of the first slot
    // loaded (`head`); then head + own continues in the accumulators.  Same additions, same order, same operands as
    // adding up all S slots one after the other.
    const int mine = P.join_slot, others = S - 1;
#pragma unroll
    for (int qt = 0; qt < 4; ++qt) {
      u32x4_t in[3][8];
      bool folded = mine == 0;                    // the accumulators already hold the running sum
      auto fetch = [&](int d, int other) {        // slot number of the other-th of the other slots
        const int sl = other < mine ? other : other + 1;
#pragma unroll
        for (int i = 0; i < 8; ++i)
          in[d][i] = __builtin_amdgcn_raw_buffer_load_b128(slots, at, (sl << 18) + (qt * 8 + i) * 1024, kDeviceScope);   // the quad's place goes into the scalar offset: one address register for all loads
      };
      auto fold_head = [&]() {                    // head + own
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float4_t h = __builtin_bit_cast(float4_t, in[0][i]);
          const int bm = qt * 2 + (i >> 2), bn = i & 3;
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[bm][4 * bn + r] = h[r] + acc[bm][4 * bn + r];
        }
        folded = true;
      };
      auto take = [&](int d, int other) {
        const int sl = other < mine ? other : other + 1;
        if (!folded && sl > mine) fold_head();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float4_t v = __builtin_bit_cast(float4_t, in[d][i]);
          const int bm = qt * 2 + (i >> 2), bn = i & 3;
          if (folded) {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[bm][4 * bn + r] = acc[bm][4 * bn + r] + v[r];
          } else if (d != 0) {
            float4_t h = __builtin_bit_cast(float4_t, in[0][i]);
#pragma unroll
            for (int r = 0; r < 4; ++r) h[r] = h[r] + v[r];
            in[0][i] = __builtin_bit_cast(u32x4_t, h);
          }
        }
      };
      // first round trip: up to three of the others; later ones: two at a time beside the head
#pragma unroll
      for (int d = 0; d < 3; ++d)
        if (d < others) fetch(d, d);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int d = 0; d < 3; ++d)
        if (d < others) take(d, d);
      __builtin_amdgcn_sched_barrier(0);
      for (int k = 3; k < others; k += 2) {
#pragma unroll
        for (int d = 0; d < 2; ++d)
          if (k + d < others) fetch(1 + d, k + d);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < 2; ++d)
          if (k + d < others) take(1 + d, k + d);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (!folded) fold_head();                   // the own slot is the last one
    }
    __syncthreads();     // the flag's word is about to be reused as staging
  }

  timeline_stamp(rec, 5, t);
  // ---- epilogue: lane holds, for row m, columns n .. n+3 of each 16-column block
  TOut* __restrict__ Cg = static_cast<TOut*>(P.C);
  const bool vec_ok = ((P.ldc & 3) == 0) && ((reinterpret_cast<uintptr_t>(Cg) & 15) == 0);
  // the whole-tile path stores 16 bytes per lane: rows of 8 bf16 or 4 fp32 elements must keep that alignment
  const bool rows_16b = (P.ldc & (16 / static_cast<int>(sizeof(TOut)) - 1)) == 0;
  const int rows_own = m_end - m0, rows_write = m_write_end - m0;    // of the tile's 256 rows: valid, written (zeros between)
  // the last tile row of a problem also clears what the static block has below its 256-row footprint (an expert with
  // few occupied slots; at most kRowsBelow rows), over this tile's columns; what lies beyond, and the static columns
  // right of the last tile column, are cleared by the fill kernel
  if (m_end == P.Mv && m_write_end < P.Ms) {
    const int col_end = min(n0 + kMfmaBN, P.Ns);
    constexpr int kPer = 16 / static_cast<int>(sizeof(TOut));
    zero_rows_below<TOut>(Cg, P.ldc, m_write_end, rows_cleared(P.Mv, P.Ms), n0, col_end, vec_ok && rows_16b && ((col_end - n0) % kPer) == 0, t);
  }
  if (vec_ok && rows_16b) {
    // 16-byte stores of whole lines; bf16 through the hardware round-to-nearest-even conversion.  A tile with all 256
    // columns (and rows) valid stores without predicates; in the last tile column a lane's 16 bytes are masked beyond
    // the valid columns, and the chunk that the static block ends in (if it ends inside one) is stored element by
    // element, so that nothing is written beyond the block's static width.
    // Relu or not is decided once per workgroup, not per element: with the test inside the conversion loop the compiler
    // turns every element into a compare, a select and a repack.  Stores go through global-address-space pointers
    // (a flat store also counts as an LDS operation, and the waits for the staging reads would wait for it) with the
    // non-temporal hint (the output is written once and not read again by this launch; with 2 GB of output per launch
    // the hint is worth 8 %); all of a wave's staging reads are issued before its first store.
    const bool relu = epilogue == GSPMD_EPILOGUE_RELU;
    const bool all_cols = n0 + kMfmaBN <= P.Nv;
    const bool whole = rows_own >= kMfmaBM && all_cols;          // all 256 rows and columns valid: no predicates
    if constexpr (sizeof(TOut) == 2) {
      // bf16: the wave's 128 x 64 block is a 128-byte line per row, but a lane holds only 8 bytes of it per 16-column
      // block.  Stage it through the wave's own slice of LDS (free now: every wave's LDS reads are over and no tile load is in flight;
      // rows padded to 144 bytes against bank conflicts) and store 16 bytes per lane, 8 lanes per row: whole lines.
      constexpr int kPitch = 144;
      unsigned char* slice = smem + wave * (128 * kPitch);
      typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
      auto stage = [&](auto relu_tag) {
        constexpr bool kRelu = decltype(relu_tag)::value;
#pragma unroll
        for (int bm = 0; bm < 8; ++bm)
#pragma unroll
          for (int bn = 0; bn < 4; ++bn) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = apply_epilogue(acc[bm][bn * 4 + j], kRelu ? GSPMD_EPILOGUE_RELU : GSPMD_EPILOGUE_NONE);
            bf16x4_t o = {static_cast<__bf16>(v[0]), static_cast<__bf16>(v[1]), static_cast<__bf16>(v[2]), static_cast<__bf16>(v[3])};
            *reinterpret_cast<bf16x4_t*>(slice + (bm * 16 + (lane & 15)) * kPitch + bn * 32 + (lane >> 4) * 8) = o;
          }
      };
      if (relu) stage(std::true_type{}); else stage(std::false_type{});
      global_u32x4_t* c0 = (global_u32x4_t*)(Cg + static_cast<int64_t>(m0 + wm * 128 + (lane >> 3)) * P.ldc + n0 + wn * 64 + (lane & 7) * 8);
      const int64_t pitch8 = static_cast<int64_t>(P.ldc);      // 8 rows of bf16 in units of 16 bytes
      const int row0 = wm * 128 + (lane >> 3);
      u32x4_t v[16];
#pragma unroll
      for (int p = 0; p < 16; ++p) v[p] = *reinterpret_cast<const u32x4_t*>(slice + (p * 8 + (lane >> 3)) * kPitch + (lane & 7) * 16);
      if (whole) {
#pragma unroll
        for (int p = 0; p < 16; ++p) __builtin_nontemporal_store(v[p], &c0[p * pitch8]);
      } else if (all_cols) {
#pragma unroll
        for (int p = 0; p < 16; ++p) {
          const int row = row0 + p * 8;
          if (row >= rows_own) v[p] = u32x4_t{0u, 0u, 0u, 0u};
          if (row < rows_write) __builtin_nontemporal_store(v[p], &c0[p * pitch8]);
        }
      } else {
        const int col = n0 + wn * 64 + (lane & 7) * 8;                         // this lane's 8 columns
        const int keep = max(0, min(8, P.Nv - col)), room = max(0, min(8, P.Ns - col));
#pragma unroll
        for (int p = 0; p < 16; ++p) {
          const int row = row0 + p * 8;
          const u32x4_t o = row < rows_own ? mask_tail8(v[p], keep) : u32x4_t{0u, 0u, 0u, 0u};
          if (row >= rows_write) continue;
          if (room == 8) {
            __builtin_nontemporal_store(o, &c0[p * pitch8]);
          } else {
            bf16_bits* out = reinterpret_cast<bf16_bits*>(Cg) + static_cast<int64_t>(m0 + row) * P.ldc + col;
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (e < room) out[e] = static_cast<bf16_bits>(o[e >> 1] >> ((e & 1) * 16));
          }
        }
      }
    } else {
      // fp32: a row of the wave's block is 256 bytes, of which a lane holds 16 per 16-column block.  Staged through the
      // wave's LDS slice in two passes of 64 rows (rows padded to 272 bytes) and stored 16 lanes per row: whole rows.
      constexpr int kPitch = 272;
      unsigned char* slice = smem + wave * (128 * 144);
      global_u32x4_t* c0 = (global_u32x4_t*)(Cg + static_cast<int64_t>(m0 + wm * 128 + (lane >> 4)) * P.ldc + n0 + wn * 64 + (lane & 15) * 4);
      const int64_t pitch4 = static_cast<int64_t>(P.ldc);      // 4 rows of fp32 in units of 16 bytes
#pragma unroll
      for (int pass = 0; pass < 2; ++pass) {
        auto stage = [&](auto relu_tag) {
          constexpr bool kRelu = decltype(relu_tag)::value;
#pragma unroll
          for (int b4 = 0; b4 < 4; ++b4) {
            const int bm = pass * 4 + b4;
#pragma unroll
            for (int bn = 0; bn < 4; ++bn) {
              float4_t v;
#pragma unroll
              for (int j = 0; j < 4; ++j) v[j] = apply_epilogue(acc[bm][bn * 4 + j], kRelu ? GSPMD_EPILOGUE_RELU : GSPMD_EPILOGUE_NONE);
              *reinterpret_cast<float4_t*>(slice + (b4 * 16 + (lane & 15)) * kPitch + bn * 64 + (lane >> 4) * 16) = v;
            }
          }
        };
        if (relu) stage(std::true_type{}); else stage(std::false_type{});
        u32x4_t v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = *reinterpret_cast<const u32x4_t*>(slice + (i * 4 + (lane >> 4)) * kPitch + (lane & 15) * 16);
        if (whole) {
#pragma unroll
          for (int i = 0; i < 16; ++i) __builtin_nontemporal_store(v[i], &c0[(pass * 16 + i) * pitch4]);
        } else if (all_cols) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row = wm * 128 + pass * 64 + i * 4 + (lane >> 4);
            if (row >= rows_own) v[i] = u32x4_t{0u, 0u, 0u, 0u};
            if (row < rows_write) __builtin_nontemporal_store(v[i], &c0[(pass * 16 + i) * pitch4]);
          }
        } else {
          const int col = n0 + wn * 64 + (lane & 15) * 4;                      // this lane's 4 columns
          const int keep = max(0, min(4, P.Nv - col)), room = max(0, min(4, P.Ns - col));
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row = wm * 128 + pass * 64 + i * 4 + (lane >> 4);
            u32x4_t o = v[i];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (row >= rows_own || e >= keep) o[e] = 0u;
            if (row >= rows_write) continue;
            if (room == 4) {
              __builtin_nontemporal_store(o, &c0[(pass * 16 + i) * pitch4]);
            } else {
              uint32_t* out = reinterpret_cast<uint32_t*>(Cg) + static_cast<int64_t>(m0 + row) * P.ldc + col;
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (e < room) out[e] = o[e];
            }
          }
        }
      }
    }
    if (rec != nullptr) {
      timeline_stamp(rec, 6, t);
      GSPMD_WAIT_ALL();
      timeline_stamp(rec, 7, t);
    }
    return;
  }
#pragma unroll
  for (int bm = 0; bm < 8; ++bm) {
    const int m = m0 + wm * 128 + bm * 16 + (lane & 15);
    if (m >= m_write_end) continue;
    const bool mrow = m < m_end;
    TOut* crow = Cg + static_cast<int64_t>(m) * P.ldc;
#pragma unroll
    for (int bn = 0; bn < 4; ++bn) {
      const int n = n0 + wn * 64 + bn * 16 + (lane >> 4) * 4;
      if (n >= P.Ns) continue;
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = (mrow && n + j < P.Nv) ? apply_epilogue(acc[bm][bn * 4 + j], epilogue) : 0.f;
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
  if (rec != nullptr) {
    timeline_stamp(rec, 6, t);
    GSPMD_WAIT_ALL();
    timeline_stamp(rec, 7, t);
  }
}

constexpr int kMaxDevices = 64;

// The kernel needs all 160 KiB of LDS as dynamic shared memory: raised once per instantiation and device.  Callable
// from several host threads.
template <typename TOut, int LAYOUT, bool STAGED>
inline bool launch_dot_mfma_as(const InlineProblems& inl, const Problem* tab, int n_prob, int tiles, int epilogue, float* join_partials,
                               uint32_t* join_counters, unsigned long long* timeline, int timeline_records, hipStream_t stream) {
  static std::once_flag once[kMaxDevices];
  static bool ok[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
  std::call_once(once[dev], [dev] {
    ok[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(&dot_mfma_kernel<TOut, LAYOUT, STAGED>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLds) == hipSuccess;
  });
  if (!ok[dev]) return false;
  const dim3 grid(static_cast<unsigned>(tiles)), block(kMfmaThreads);
  hipLaunchKernelGGL((dot_mfma_kernel<TOut, LAYOUT, STAGED>), grid, block, kMfmaLds, stream, inl, tab, n_prob, epilogue, join_partials, join_counters,
                     timeline, timeline_records);
  return hipGetLastError() == hipSuccess;
}

template <typename TOut, bool STAGED>
inline bool launch_dot_mfma_layout(const InlineProblems& inl, const Problem* tab, int n_prob, int tiles, int32_t layout, int epilogue,
                                   float* join_partials, uint32_t* join_counters, unsigned long long* timeline, int timeline_records,
                                   hipStream_t stream) {
  switch (layout & 3) {
    case 0: return launch_dot_mfma_as<TOut, 0, STAGED>(inl, tab, n_prob, tiles, epilogue, join_partials, join_counters, timeline, timeline_records, stream);
    case 1: return launch_dot_mfma_as<TOut, 1, STAGED>(inl, tab, n_prob, tiles, epilogue, join_partials, join_counters, timeline, timeline_records, stream);
    case 2: return launch_dot_mfma_as<TOut, 2, STAGED>(inl, tab, n_prob, tiles, epilogue, join_partials, join_counters, timeline, timeline_records, stream);
    default: return launch_dot_mfma_as<TOut, 3, STAGED>(inl, tab, n_prob, tiles, epilogue, join_partials, join_counters, timeline, timeline_records, stream);
  }
}

// `staged`: the operands allow 4-byte but not 16-byte aligned chunk loads
inline bool launch_dot_mfma(const InlineProblems& inl, const Problem* tab, int n_prob, int tiles, int32_t layout, int32_t out_dtype,
                            bool staged, int epilogue, float* join_partials, uint32_t* join_counters, unsigned long long* timeline,
                            int timeline_records, hipStream_t stream) {
  const bool f32 = out_dtype == GSPMD_F32;
  if (staged)
    return f32 ? launch_dot_mfma_layout<float, true>(inl, tab, n_prob, tiles, layout, epilogue, join_partials, join_counters, timeline, timeline_records, stream)
               : launch_dot_mfma_layout<bf16_bits, true>(inl, tab, n_prob, tiles, layout, epilogue, join_partials, join_counters, timeline, timeline_records, stream);
  return f32 ? launch_dot_mfma_layout<float, false>(inl, tab, n_prob, tiles, layout, epilogue, join_partials, join_counters, timeline, timeline_records, stream)
             : launch_dot_mfma_layout<bf16_bits, false>(inl, tab, n_prob, tiles, layout, epilogue, join_partials, join_counters, timeline, timeline_records, stream);
}

}  // namespace gspmd
