/* A C99 program that runs the tiny 1-D sharded matmul (A[8,64] x B[64,90], N split over 4 partitions: shards of 23
 * columns, the last holding 21, Section 4.1) on the GPU through the C ABI alone: shard bounds, DynamicSlice of the rhs
 * into poisoned shard buffers, one gspmd_local_dot per partition, DynamicUpdateSlice of the out shards.  Operands are
 * read from a file written by tests/test_gpu_c_abi.py, the reassembled product is written back for the test to compare
 * with the oracle; nothing here knows of Python or torch.
 * usage: c_device_check <in: 8*64 + 64*90 floats> <out: 8*90 floats> */
#include <stdio.h>
#include <stdlib.h>
#include <hip/hip_runtime_api.h>
#include "gspmd.h"

#define M 8
#define K 64
#define N 90
#define P 4

static int fail(const char* what, int code) {
  fprintf(stderr, "c_device_check: %s (%d)\n", what, code);
  return 1;
}

int main(int argc, char** argv) {
  if (argc != 3) return fail("usage", 0);
  static float a[M * K], b[K * N], c[M * N];
  FILE* f = fopen(argv[1], "rb");
  if (!f || fread(a, sizeof(float), M * K, f) != M * K || fread(b, sizeof(float), K * N, f) != K * N) return fail("read", 0);
  fclose(f);

  const int64_t mesh_shape[1] = {P}, ids[P] = {2, 0, 3, 1};
  const gspmd_mesh mesh = {1, mesh_shape, ids};
  const int64_t ls[2] = {M, K}, rs[2] = {K, N}, os[2] = {M, N};
  const int32_t lm[2] = {-1, -1}, rm[2] = {-1, 0}, om[2] = {-1, 0};
  const gspmd_sharding lsh = {2, ls, lm}, rsh = {2, rs, rm}, osh = {2, os, om};
  const int32_t lc[1] = {1}, rc[1] = {0};
  const gspmd_dot_dims dims = {0, NULL, NULL, 1, lc, rc};

  int64_t off[2], valid[2], shard[2];
  if (gspmd_shard_bounds(&mesh, &rsh, 0, off, valid, shard) != GSPMD_OK) return fail("bounds", 0);
  if (shard[1] != 23) return fail("static shard size", (int)shard[1]);

  float *da, *db, *dc, *drs[P], *dos[P];
  void* ws;
  int64_t ws_bytes = 0;
  hipError_t e;
  if ((e = hipMalloc((void**)&da, sizeof(a))) != hipSuccess || (e = hipMalloc((void**)&db, sizeof(b))) != hipSuccess ||
      (e = hipMalloc((void**)&dc, sizeof(c))) != hipSuccess) return fail("hipMalloc", (int)e);
  if ((e = hipMemcpy(da, a, sizeof(a), hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipMemcpy(db, b, sizeof(b), hipMemcpyHostToDevice)) != hipSuccess) return fail("hipMemcpy", (int)e);
  if ((e = hipMemset(dc, 0xff, sizeof(c))) != hipSuccess) return fail("hipMemset", (int)e);   /* NaN until written */
  int32_t st = gspmd_dot_workspace_bytes(&mesh, &dims, &lsh, &rsh, &osh, 0, 0, &ws_bytes);
  if (st != GSPMD_OK) return fail(gspmd_status_string(st), st);
  if ((e = hipMalloc(&ws, (size_t)ws_bytes + 256)) != hipSuccess) return fail("hipMalloc", (int)e);
  void* ws_aligned = (void*)(((uintptr_t)ws + 255) / 256 * 256);

  const gspmd_shard_buf lhs = {da, GSPMD_F32, 0};
  for (int p = 0; p < P; ++p) {
    if (hipMalloc((void**)&drs[p], K * 23 * sizeof(float)) != hipSuccess || hipMalloc((void**)&dos[p], M * 23 * sizeof(float)) != hipSuccess)
      return fail("hipMalloc", p);
    const gspmd_shard_buf rhs = {drs[p], GSPMD_F32, 0}, out = {dos[p], GSPMD_F32, 0};
    /* padding of the rhs shard is poisoned with NaN; it must not reach the product */
    if ((st = gspmd_shard_extract(&mesh, &rsh, p, db, &rhs, 0x7FC00000u, NULL)) != GSPMD_OK) return fail(gspmd_status_string(st), st);
    if ((st = gspmd_local_dot(&mesh, &dims, &lhs, &lsh, &rhs, &rsh, &out, &osh, p, NULL, GSPMD_EPILOGUE_NONE, ws_aligned, ws_bytes,
                              NULL)) != GSPMD_OK)
      return fail(gspmd_status_string(st), st);
    if ((st = gspmd_shard_assemble(&mesh, &osh, p, &out, dc, NULL)) != GSPMD_OK) return fail(gspmd_status_string(st), st);
  }
  if ((e = hipDeviceSynchronize()) != hipSuccess) return fail("hipDeviceSynchronize", (int)e);
  if ((e = hipMemcpy(c, dc, sizeof(c), hipMemcpyDeviceToHost)) != hipSuccess) return fail("hipMemcpy", (int)e);
  /* the partition in mesh position 3 (id 1) holds 21 valid columns; its out shard's padding must be zero */
  static float last[M * 23];
  if (hipMemcpy(last, dos[1], sizeof(last), hipMemcpyDeviceToHost) != hipSuccess) return fail("hipMemcpy", 0);
  for (int m = 0; m < M; ++m)
    for (int n = 21; n < 23; ++n)
      if (last[m * 23 + n] != 0.0f) return fail("padding of the last out shard is not zero", m);
  f = fopen(argv[2], "wb");
  if (!f || fwrite(c, sizeof(float), M * N, f) != M * N) return fail("write", 0);
  fclose(f);
  puts("c device ok");
  return 0;
}
