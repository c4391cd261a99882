// Integer index math of the MFMA kernel's tiles: which output tile a workgroup takes, where every lane of a tile
// load reads in global memory and where its 16 bytes land in LDS, and where every lane reads its fragments.  Kept
// apart from the kernel, and callable on the host, so that tests can check on the CPU that loads and fragment reads
// agree and that no load leaves the valid extents.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define GSPMD_INDEX_FN __host__ __device__ __forceinline__

namespace gspmd {

constexpr int kMfmaBM = 256, kMfmaBN = 256, kMfmaBK = 32;
constexpr int kMfmaThreads = 512;
constexpr int kStageA = kMfmaBM * kMfmaBK * 2;     // 16 KiB
constexpr int kStageB = kMfmaBK * kMfmaBN * 2;     // 16 KiB
constexpr int kStage = kStageA + kStageB;
constexpr int kNumStages = 5;
constexpr int kMfmaLds = kNumStages * kStage;      // all 160 KiB of the CU's LDS

GSPMD_INDEX_FN int swz_a(int row) { return (row >> 1) & 3; }
GSPMD_INDEX_FN int swz_b(int krow) { return ((krow & 3) << 2) ^ (((krow >> 3) & 1) << 1); }

// Which output tile a workgroup takes.  Workgroup b runs on XCD b % 8 (each XCD has its own L2), and 256
// workgroups are resident at a time.  Within every window of 256 consecutive tile ids (the last window may be
// shorter) XCD x takes a run of consecutive ids -- [32x, 32x+32) of a full window, an eighth of a short one -- and
// inside a problem ids walk bands of 8 tile rows with the row index running fastest: an XCD's 32 concurrent tiles
// then form a block of about 8 rows x 4 columns (12 operand panels per K step instead of up to 33), and a problem
// with few tile rows (an expert with <= 1024 occupied slots) streams every weight panel exactly once, all its row
// tiles being in flight together.
GSPMD_INDEX_FN int logical_tile(int b, int total) {
  const int base = b & ~255;
  const int left = total - base;
  const int width = left < 256 ? left : 256;       // ids in this window
  const int r = b - base, x = r & 7, i = r >> 3;    // XCD x, its i-th workgroup of the window
  const int each = width >> 3, extra = width & 7;   // XCDs 0 .. extra-1 have one workgroup more
  return base + x * each + (x < extra ? x : extra) + i;
}

constexpr int kBandRows = 8;

GSPMD_INDEX_FN int swz_h(int row) { return (row >> 1) & 7; }

// Main loop, K-contiguous operand: part `half` (0/1) of a 64-wide K step is [128 rows][64 k] with 128-byte rows.
// Per-lane byte offset, relative to the address of (first row of the 256-row tile, first k of the step), of load
// instruction q (0..15; rows 8q..8q+7 of the half, 8 lanes per row).  Rows past the valid extent reuse the last
// valid row (their results are never stored).
GSPMD_INDEX_FN int kc_half_load_offset(int q, int lane, int half, int r0, int rows_valid, int ld) {
  const int r = q * 8 + (lane >> 3);
  const int c = (lane & 7) ^ swz_h(r);
  const int last = rows_valid - 1, want = r0 + half * 128 + r;
  const int rr = (want < last ? want : last) - r0;
  return (rr * ld + c * 8) * 2;
}
// LDS byte offset inside the part of a lane's first fragment (first 32 k of the step; the second at ^ 64) of the
// 16-row block whose first row inside the half is `base`; block b at + b * 2048.
GSPMD_INDEX_FN int kc_half_frag_offset(int base, int lane) {
  const int row = base + (lane & 15);
  return row * 128 + (((lane >> 4) ^ swz_h(row)) << 4);
}

// What is left of K after the main loop uses [256 rows][32 k] parts for a K-contiguous operand:
// per-lane byte offset, relative to the tile's base, of load instruction q (0..15) of a K-contiguous operand tile
// ([256 rows][32 k]: instruction q covers rows 16q..16q+15, 4 lanes per row).  Rows past the valid extent reuse the
// last valid row (their results are never stored).
GSPMD_INDEX_FN int kc_load_offset(int q, int lane, int r0, int rows_valid, int ld) {
  const int r = q * 16 + (lane >> 2);
  const int c = (lane & 3) ^ swz_a(r);
  const int last = rows_valid - 1, want = r0 + r;
  const int rr = (want < last ? want : last) - r0;
  return (rr * ld + c * 8) * 2;
}
// Same for a K-major operand tile ([32 k][256 columns]: instruction q covers k rows 2q, 2q+1, 32 lanes per row).
// 16-byte chunks past the valid extent reuse the last valid chunk.
GSPMD_INDEX_FN int km_load_offset(int q, int lane, int c0, int cols_valid, int ld) {
  const int kr = q * 2 + (lane >> 5);
  const int cn = (lane & 31) ^ swz_b(kr);
  int n = c0 + cn * 8;
  if (n >= cols_valid) n = ((cols_valid - 1) >> 3) << 3;
  return (kr * ld + (n - c0)) * 2;
}
// LDS byte offset (inside the operand's part of a stage) of a lane's fragment of 16-row block 0 whose first row is
// `base`: K-contiguous tile, block b at + b * 1024.
GSPMD_INDEX_FN int kc_frag_offset(int base, int lane) {
  const int row = base + (lane & 15);
  return row * 64 + (((lane >> 4) ^ swz_a(row)) << 4);
}
// K-major tile (read with the transpose read): block b at ^ (b << 5), second half of the fragment at + 4 * 512.
GSPMD_INDEX_FN int km_frag_offset(int base, int lane) {
  const int i = lane & 15;
  const int krow = (lane >> 4) * 8 + (i >> 2);
  const int cl = base + (i & 3) * 4;
  return krow * 512 + (((cl >> 3) ^ swz_b(krow)) << 4) + (cl & 7) * 2;
}

// How the valid rows of a problem are divided among its tile rows.  The work of a tile is proportional to the
// 16-row blocks it multiplies, and workgroups are handed to compute units in id order, so a launch finishes soonest
// when its tiles cost about the same: the ceil(rows / 16) blocks are split as evenly as possible over the
// ceil(rows / 256) tile rows (the first `extra` tile rows take one block more), instead of whole 256-row tiles and one
// short one.  Tile row i owns rows [first, first + rows) of the problem; only the last tile row can own a number of
// rows that is not a multiple of 16.
struct TileRows {
  int first;   // first row the tile owns
  int rows;    // valid rows it owns (1..256)
};
GSPMD_INDEX_FN TileRows tile_rows(int i, int rows_valid) {
  const int tiles_m = (rows_valid + kMfmaBM - 1) / kMfmaBM;
  const int blocks = (rows_valid + 15) >> 4;
  const int base = blocks / tiles_m, extra = blocks - base * tiles_m;
  TileRows t;
  t.first = (i * base + (i < extra ? i : extra)) * 16;
  const int own = (base + (i < extra ? 1 : 0)) * 16;
  t.rows = (i == tiles_m - 1) ? rows_valid - t.first : own;
  return t;
}
// Rows of a problem's static output block that its tiles write (valid rows, then zeros up to the end of the last
// tile's 256-row footprint); what lies beyond is zero-filled apart.
GSPMD_INDEX_FN int rows_written(int rows_valid, int rows_static) {
  if (rows_valid <= 0) return 0;
  const int tiles_m = (rows_valid + kMfmaBM - 1) / kMfmaBM;
  const int end = tile_rows(tiles_m - 1, rows_valid).first + kMfmaBM;
  return end < rows_static ? end : rows_static;
}

// Rows of the static output block that the workgroups of a problem's last tile row clear in all: their own footprint
// and up to kRowsBelow rows below it (an expert with few occupied slots).  A block that goes on beyond that is
// cleared by the fill kernel, which spreads the work over the whole chip.
constexpr int kRowsBelow = 1024;
GSPMD_INDEX_FN int rows_cleared(int rows_valid, int rows_static) {
  const int written = rows_written(rows_valid, rows_static);
  if (written <= 0) return 0;
  return rows_static - written <= kRowsBelow ? rows_static : written + kRowsBelow;
}

// Tile `local` (0-based inside its problem) of a problem with `rows_valid` valid rows and `tiles_n` tile columns: its
// tile row and its first column.  Ids walk bands of kBandRows tile rows, the row index running fastest inside a band.
GSPMD_INDEX_FN void tile_origin(int local, int rows_valid, int tiles_n, int* tile_row, int* n0) {
  const int tiles_m = (rows_valid + kMfmaBM - 1) / kMfmaBM;   // tiles cover the valid extents; the rest of the static block is zero-filled apart
  const int band = local / (kBandRows * tiles_n);
  const int left = tiles_m - band * kBandRows;
  const int rows_in_band = left < kBandRows ? left : kBandRows;
  const int in_band = local - band * kBandRows * tiles_n;
  *tile_row = band * kBandRows + in_band % rows_in_band;
  *n0 = (in_band / rows_in_band) * kMfmaBN;
}

}  // namespace gspmd
