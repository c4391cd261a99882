/* Compiled as C99 by tests/test_c_abi.py against include/gspmd.h and linked with libgspmd.so: the header must be plain C
 * and the host-only entry points must work from a program that knows nothing of Python or torch.  Values checked are
 * the paper's: a dimension of 90 split 4 ways has shards of 23 with the last one holding 21 (Section 4.1), and the
 * BD,DF->BF example of Section 3.2 is data parallel on mesh dimension 0 and model parallel on mesh dimension 1. */
#include <stdio.h>
#include <string.h>
#include "gspmd.h"

int main(void) {
  const int64_t mesh_shape[1] = {4}, ids[4] = {2, 0, 3, 1};
  gspmd_mesh mesh = {1, mesh_shape, ids};
  const int64_t shape[2] = {8, 90};
  const int32_t map[2] = {-1, 0};
  gspmd_sharding sh = {2, shape, map};
  int64_t off[2], valid[2], shard[2];
  /* device 1 sits at mesh position 3: offset 69, 21 valid of 23 */
  if (gspmd_shard_bounds(&mesh, &sh, 1, off, valid, shard) != GSPMD_OK) return 1;
  if (off[0] != 0 || valid[0] != 8 || shard[0] != 8 || off[1] != 69 || valid[1] != 21 || shard[1] != 23) return 2;
  if (gspmd_shard_bounds(&mesh, &sh, 4, off, valid, shard) != GSPMD_ERR_PARTITION_RANGE) return 3;
  if (gspmd_shard_bounds(NULL, &sh, 0, off, valid, shard) != GSPMD_ERR_NULL) return 4;

  const int64_t mesh2_shape[2] = {2, 2}, ids2[4] = {0, 1, 2, 3};
  gspmd_mesh mesh2 = {2, mesh2_shape, ids2};
  const int32_t lc[1] = {1}, rc[1] = {0};
  gspmd_dot_dims dims = {0, NULL, NULL, 1, lc, rc};
  const int64_t ls[2] = {64, 32}, rs[2] = {32, 48}, os[2] = {64, 48};
  const int32_t lm[2] = {0, -1}, rm[2] = {-1, 1}, om[2] = {0, 1};
  gspmd_sharding lsh = {2, ls, lm}, rsh = {2, rs, rm}, osh = {2, os, om};
  int32_t cls[2];
  if (gspmd_classify_dot(&mesh2, &dims, &lsh, &rsh, &osh, cls) != GSPMD_OK) return 5;
  if (cls[0] != GSPMD_AXIS_LHS_FREE || cls[1] != GSPMD_AXIS_RHS_FREE) return 6;
  int32_t inferred[2], rank = 0;
  int64_t oshape[2];
  if (gspmd_infer_out_sharding(&mesh2, &dims, &lsh, &rsh, inferred, oshape, &rank) != GSPMD_OK) return 7;
  if (rank != 2 || inferred[0] != 0 || inferred[1] != 1 || oshape[0] != 64 || oshape[1] != 48) return 8;
  gspmd_gemm_desc d;
  int64_t count = 0;
  if (gspmd_plan_dot(&mesh2, &dims, &lsh, &rsh, &osh, 0, 0, 0, 3, NULL, &d, 1, &count) != GSPMD_OK) return 9;
  if (count != 1 || d.m_valid != 32 || d.n_valid != 24 || d.k_valid != 32 || d.layout != 0) return 10;
  int64_t bytes = 0;
  if (gspmd_dot_workspace_bytes(&mesh2, &dims, &lsh, &rsh, &osh, -1, 0, &bytes) != GSPMD_OK || bytes <= 0) return 11;
  if (gspmd_reshard_workspace_bytes(&mesh2, &bytes) != GSPMD_OK || bytes <= 0) return 12;
  if (strcmp(gspmd_status_string(GSPMD_ERR_NEEDS_RESHARD), "shardings need resharding") != 0) return 13;
  puts("c abi ok");
  return 0;
}
