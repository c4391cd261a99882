// Host-side check of csrc/tile_index.h (built and run by tests/test_tile_index.py; no GPU is touched).
// A tile load writes lane i's 16 bytes at (instruction's LDS base + 16 i); the per-lane global offsets decide which
// element lands where.  For every tile format this program replays the loads into a map LDS byte -> (row, k) or
// (k, column), replays the fragment reads (plain 16-byte reads and the 4 x 16 transpose read) and compares what each
// lane receives with the operand layout of v_mfma_f32_16x16x32_bf16 (lane l: row or column l & 15, k = 8 (l >> 4) .. + 7).
// It also checks that no load offset leaves the valid rows / 16-byte chunks, and that the tile order visits every tile
// of a problem, and every workgroup id of a launch, exactly once.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <utility>
#include <vector>

#include "../paper_2105_04663_amd/csrc/tile_index.h"

using namespace gspmd;

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (failures < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++failures; } } while (0)

typedef std::pair<int, int> RC;                 // (row, k) of a K-contiguous part, (k, column) of a K-major part

// ---- K-contiguous operand, main loop: half h of a 64-wide step as [128 rows][64 k]
static void check_kc_half(int r0, int rows_valid, int ld) {
  for (int h = 0; h < 2; ++h) {
    std::map<int, RC> lds;                      // byte offset in the part -> element
    for (int q = 0; q < 16; ++q)
      for (int lane = 0; lane < 64; ++lane) {
        const int off = kc_half_load_offset(q, lane, h, r0, rows_valid, ld);
        CHECK(off >= 0 && off % 16 == 0, "kc half offset %d", off);
        const int row = (off / 2) / ld, k = (off / 2) % ld;
        CHECK(k + 8 <= 64, "kc half: k chunk %d leaves the 64-wide step", k);
        CHECK(r0 + row < rows_valid, "kc half: row %d beyond the %d valid rows (r0 %d)", r0 + row, rows_valid, r0);
        const int want_row = h * 128 + q * 8 + (lane >> 3);
        if (r0 + want_row < rows_valid) CHECK(row == want_row, "kc half: row %d instead of %d", row, want_row);
        for (int e = 0; e < 8; ++e) lds[q * 1024 + lane * 16 + 2 * e] = RC(row, k + e);
      }
    CHECK(lds.size() == 128 * 64, "kc half: %zu elements", lds.size());
    // fragment reads: block b of 16 rows at + 2048 b, the step's second 32 k at ^ 64; any first row that is a multiple
    // of 16 inside a 64-row group of the half (the kernel uses 0 for the lhs and 0 / 64 for the rhs)
    for (int base : {0, 64})
      for (int b = 0; b < (base ? 4 : 8); ++b)
        for (int q = 0; q < 2; ++q)
          for (int lane = 0; lane < 64; ++lane) {
            const int addr = (kc_half_frag_offset(base, lane) ^ (q * 64)) + b * 2048;
            for (int e = 0; e < 8; ++e) {
              const RC got = lds.at(addr + 2 * e);
              const int want_row = h * 128 + base + b * 16 + (lane & 15), want_k = q * 32 + (lane >> 4) * 8 + e;
              if (r0 + want_row < rows_valid) CHECK(got.first == want_row, "kc half read: row %d instead of %d", got.first, want_row);
              CHECK(got.second == want_k, "kc half read: k %d instead of %d", got.second, want_k);
            }
          }
  }
}

// ---- K-contiguous operand, what is left of K: [256 rows][32 k]
static void check_kc_tail(int r0, int rows_valid, int ld) {
  std::map<int, RC> lds;
  for (int q = 0; q < 16; ++q)
    for (int lane = 0; lane < 64; ++lane) {
      const int off = kc_load_offset(q, lane, r0, rows_valid, ld);
      CHECK(off >= 0 && off % 16 == 0, "kc offset %d", off);
      const int row = (off / 2) / ld, k = (off / 2) % ld;
      CHECK(k + 8 <= 32 && r0 + row < rows_valid, "kc tail: row %d k %d", row, k);
      if (r0 + q * 16 + (lane >> 2) < rows_valid) CHECK(row == q * 16 + (lane >> 2), "kc tail: row %d", row);
      for (int e = 0; e < 8; ++e) lds[q * 1024 + lane * 16 + 2 * e] = RC(row, k + e);
    }
  CHECK(lds.size() == 256 * 32, "kc tail: %zu elements", lds.size());
  for (int base : {0, 128})
    for (int b = 0; b < 8; ++b)
      for (int lane = 0; lane < 64; ++lane) {
        const int addr = kc_frag_offset(base, lane) + b * 1024;
        for (int e = 0; e < 8; ++e) {
          const RC got = lds.at(addr + 2 * e);
          const int want_row = base + b * 16 + (lane & 15);
          if (r0 + want_row < rows_valid) CHECK(got.first == want_row, "kc tail read: row %d instead of %d", got.first, want_row);
          CHECK(got.second == (lane >> 4) * 8 + e, "kc tail read: k %d", got.second);
        }
      }
}

// ---- K-major operand (main loop and tail alike): [32 k][256 columns], read with the 4 x 16 transpose read
static void check_km(int c0, int cols_valid, int ld) {
  std::map<int, RC> lds;
  const int last_chunk = ((cols_valid - 1) >> 3) << 3;
  for (int q = 0; q < 16; ++q)
    for (int lane = 0; lane < 64; ++lane) {
      const int off = km_load_offset(q, lane, c0, cols_valid, ld);
      CHECK(off >= 0 && off % 16 == 0, "km offset %d", off);
      const int kr = (off / 2) / ld, col = (off / 2) % ld;
      CHECK(kr == q * 2 + (lane >> 5), "km: k row %d", kr);
      CHECK(c0 + col <= last_chunk, "km: chunk at column %d beyond the last valid chunk %d", c0 + col, last_chunk);
      for (int e = 0; e < 8; ++e) lds[q * 1024 + lane * 16 + 2 * e] = RC(kr, col + e);
    }
  CHECK(lds.size() == 32 * 256, "km: %zu elements", lds.size());
  for (int base : {0, 64, 128, 192})            // first column of a wave's 64 (rhs) or 128 (lhs: 0, 128) columns
    for (int b = 0; b < ((base & 64) ? 4 : 8); ++b)
      for (int rd = 0; rd < 2; ++rd)
        for (int lane = 0; lane < 64; ++lane) {
          const int g = lane >> 4, j = lane & 15;
          for (int r = 0; r < 4; ++r) {
            // lane (g, j) receives, as its r-th element, sub-element j & 3 of what lane (g, 4 r + (j >> 2)) addresses
            const int src = g * 16 + 4 * r + (j >> 2);
            const int addr = (km_frag_offset(base, src) ^ (b << 5)) + rd * 2048 + (j & 3) * 2;
            const RC got = lds.at(addr);
            const int want_col = base + b * 16 + j;
            CHECK(got.first == g * 8 + rd * 4 + r, "km read: k %d instead of %d", got.first, g * 8 + rd * 4 + r);
            if (c0 + want_col < cols_valid) CHECK(got.second == want_col, "km read: column %d instead of %d", got.second, want_col);
          }
        }
}

static void check_tile_order() {
  for (int rows_valid : {1, 15, 16, 17, 128, 255, 256, 257, 734, 745, 959, 967, 1024, 1500, 2049, 5000, 16384})
    for (int tiles_n : {1, 2, 5, 32, 128}) {
      const int tiles_m = (rows_valid + kMfmaBM - 1) / kMfmaBM;
      std::set<RC> seen;
      for (int local = 0; local < tiles_m * tiles_n; ++local) {
        int tr = -1, n0 = -1;
        tile_origin(local, rows_valid, tiles_n, &tr, &n0);
        CHECK(tr >= 0 && tr < tiles_m && n0 >= 0 && n0 / kMfmaBN < tiles_n && n0 % kMfmaBN == 0,
              "tile_origin(%d, %d, %d) = (%d, %d)", local, rows_valid, tiles_n, tr, n0);
        seen.insert(RC(tr, n0));
      }
      CHECK(static_cast<int>(seen.size()) == tiles_m * tiles_n, "tile order visits %zu of %d tiles", seen.size(), tiles_m * tiles_n);
      // the tile rows own consecutive ranges that cover the valid rows exactly once; each starts on a 16-row block,
      // owns at most 256 rows, and their block counts differ by at most one
      int next = 0, lo = 1 << 30, hi = 0;
      for (int i = 0; i < tiles_m; ++i) {
        const TileRows t = tile_rows(i, rows_valid);
        CHECK(t.first == next && t.first % 16 == 0 && t.rows >= 1 && t.rows <= kMfmaBM, "tile_rows(%d, %d) = (%d, %d)", i, rows_valid, t.first, t.rows);
        if (i + 1 < tiles_m) CHECK(t.rows % 16 == 0, "tile row %d of %d rows owns %d rows", i, rows_valid, t.rows);
        const int blocks = (t.rows + 15) / 16;
        lo = blocks < lo ? blocks : lo;
        hi = blocks > hi ? blocks : hi;
        next = t.first + t.rows;
      }
      CHECK(next == rows_valid, "tile rows cover %d of %d rows", next, rows_valid);
      CHECK(hi - lo <= 1, "tile rows of %d rows have %d to %d blocks", rows_valid, lo, hi);
      for (int rows_static : {rows_valid, rows_valid + 1, rows_valid + 300, rows_valid + 5000}) {
        const int w = rows_written(rows_valid, rows_static);
        CHECK(w >= rows_valid && w <= rows_static && (w == rows_static || w == tile_rows(tiles_m - 1, rows_valid).first + kMfmaBM),
              "rows_written(%d, %d) = %d", rows_valid, rows_static, w);
      }
    }
  for (int total : {1, 7, 255, 256, 257, 511, 512, 960, 1792, 2048, 70000}) {
    std::set<int> seen;
    for (int b = 0; b < total; ++b) {
      const int t = logical_tile(b, total);
      CHECK(t >= 0 && t < total, "logical_tile(%d, %d) = %d", b, total, t);
      seen.insert(t);
    }
    CHECK(static_cast<int>(seen.size()) == total, "logical_tile is not a permutation for %d workgroups", total);
  }
  // within a window of 256 ids, XCD x (workgroups b with b % 8 == x) takes the 32 consecutive ids [32 x, 32 x + 32)
  for (int b = 0; b < 512; ++b) CHECK((logical_tile(b, 512) & 255) / 32 == (b & 7), "XCD %d gets tile %d", b & 7, logical_tile(b, 512));
  // rows cleared by a problem's tiles: never less than what they write, never more than 1024 rows below it, all of a
  // block that ends within those rows
  for (int valid : {0, 1, 255, 256, 257, 745, 1000, 5000})
    for (int extra : {0, 1, 23, 1024, 1025, 4000}) {
      const int stat = valid + extra, w = rows_written(valid, stat), c = rows_cleared(valid, stat);
      CHECK(c >= w && c <= stat && c - w <= kRowsBelow, "rows_cleared(%d, %d) = %d, written %d", valid, stat, c, w);
      CHECK(valid == 0 ? c == 0 : (stat - w <= kRowsBelow ? c == stat : c == w + kRowsBelow), "rows_cleared(%d, %d) = %d", valid, stat, c);
    }
  // a short last window is shared out the same way: the ids of one XCD are consecutive, XCD 0's first
  for (int total : {1, 5, 8, 13, 192, 255, 256 + 192, 512 + 77}) {
    const int base = total & ~255, width = total - base;
    int next = base;
    for (int x = 0; x < 8; ++x)
      for (int b = base + x; b < total; b += 8) {
        CHECK(logical_tile(b, total) == next, "short window: workgroup %d of %d gets tile %d, expected %d", b, total, logical_tile(b, total), next);
        ++next;
      }
    CHECK(next == base + width, "short window of %d ids not covered", width);
  }
}

int main() {
  for (int ld : {64, 72, 8192, 1 << 21})
    for (int r0 : {0, 256, 1024})
      for (int rows_valid : {r0 + 1, r0 + 2, r0 + 17, r0 + 127, r0 + 128, r0 + 129, r0 + 200, r0 + 255, r0 + 256, r0 + 10000}) {
        check_kc_half(r0, rows_valid, ld);
        if (ld >= 32) check_kc_tail(r0, rows_valid, ld);
      }
  for (int ld : {256, 264, 1256, 32768, 1 << 23})
    for (int c0 : {0, 256, 1024})
      for (int cols_valid : {c0 + 1, c0 + 7, c0 + 8, c0 + 9, c0 + 226, c0 + 255, c0 + 256, c0 + 9999})
        if (((cols_valid + 7) & ~7) <= ld) check_km(c0, cols_valid, ld);
  check_tile_order();
  if (failures) { printf("%d failures\n", failures); return 1; }
  printf("tile index ok\n");
  return 0;
}
