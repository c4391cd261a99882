// Host-side index math of the per-partition Dot: mesh coordinates, shard bounds
// (Section 3.5 Offset with the static shard size of Section 4.1), per-mesh-dimension
// classification of a Dot (Section 4.4) and the lowering of one partition's local Dot to a
// list of strided GEMM problems for the device kernels.  No HIP in this file.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/gspmd.h"

namespace gspmd {

// One strided GEMM the device kernels run:  C[m,n] = sum_k A[m,k] * B[k,n]  for
// m < Mv, n < Nv, k < Kv; C is written as 0 for the rest of [Ms, Ns].
// 80 bytes; the device reads an array of these.  Which index of A and of B is the contiguous
// one is the same for every problem of a launch (it follows from the Dot's dimension order)
// and travels beside the table as a mask of GSPMD_LAYOUT_* bits.
// Joined problems: join_count > 1 problems of one launch that have the same output block (C, extents) and differ in
// what they contract over -- the partitions along a contracting mesh dimension (Section 4.2), or pieces of one K
// range -- each contribute a partial sum to every output tile; the contributions are added in ascending join_slot.
struct Problem {
  const void* A;      // element (m,k) at A + m*lda + k;  lhs K-major: A + k*lda + m
  const void* B;      // element (k,n) at B + k*ldb + n;  rhs K-contiguous: B + n*ldb + k
  void* C;            // element (m,n) at C + m*ldc + n
  int32_t Mv, Nv, Kv; // valid extents (what is read / computed)
  int32_t Ms, Ns;     // static extents of the output block (zero-filled beyond valid)
  int32_t lda, ldb, ldc;
  int32_t tile_begin; // id of this problem's first output tile in the launch
  int32_t tiles_n;    // tile columns of this problem (tiles cover the valid extents only)
  int32_t join_count; // contributions per output tile; 0 or 1: this problem alone
  int32_t join_slot;  // this problem's place in the order of summation
  int32_t join_first; // index, among all joined output tiles of the launch, of this problem's tile 0
  int32_t pad;
};
static_assert(sizeof(Problem) == 80, "device layout");

// A rectangle of a problem's static output block that no output tile covers (whole tile rows / columns beyond the
// valid extents): written as 0 by a fill kernel, so that the contraction kernel is launched over live tiles only.
struct ZeroRect {
  void* C;
  int32_t ldc;
  int32_t r0, r1, c0, c1;   // rows [r0, r1) x columns [c0, c1)
  int32_t pad;
};
static_assert(sizeof(ZeroRect) == 32, "device layout");

// bytes of the launch tables per problem: the problem itself and at most two zero rectangles
constexpr int64_t kTableBytesPerProblem = sizeof(Problem) + 2 * sizeof(ZeroRect);

constexpr int kMaxRank = 8;
constexpr int64_t kMaxProblems = 1 << 20;
constexpr int64_t kMaxPartitions = 1 << 20;

struct Bounds {
  int rank = 0;
  int64_t offset[kMaxRank], valid[kMaxRank], shard[kMaxRank];
};

int32_t validate_mesh(const gspmd_mesh* mesh, int64_t* n_partitions);
int32_t validate_sharding(const gspmd_mesh* mesh, const gspmd_sharding* sh);
// Coordinates of `pid` in the row-major device tensor.
int32_t mesh_coords(const gspmd_mesh* mesh, int64_t pid, int64_t* coords);
int32_t shard_bounds(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid, Bounds* b);

// Roles of the dimensions of one Dot after validation.
struct DotRoles {
  int nb = 0, nc = 0, nlf = 0, nrf = 0;
  int lhs_free[kMaxRank], rhs_free[kMaxRank];
  int lhs_contract[kMaxRank], rhs_contract[kMaxRank]; // pairs, sorted by lhs dim
  int lhs_batch[kMaxRank], rhs_batch[kMaxRank];
};

int32_t analyse_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                    const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                    const gspmd_sharding* out_sh, DotRoles* roles, int32_t* axis_class);

// Append the GEMM problems of partition `pid` to `out` (tile fields left 0).
// `c_override`/`c_dtype`: when non-null the output goes to a dense fp32 partial buffer
// instead of the partition's out shard.
int32_t plan_partition(const gspmd_mesh* mesh, const DotRoles& roles,
                       const gspmd_shard_buf* lhs, const gspmd_sharding* lhs_sh,
                       const gspmd_shard_buf* rhs, const gspmd_sharding* rhs_sh,
                       const gspmd_shard_buf* out, const gspmd_sharding* out_sh,
                       int64_t pid, const int64_t* lhs_fill, void* c_override,
                       std::vector<Problem>* problems, int64_t* out_static_elems, int32_t* layout);

// Upper bound of the number of problems plan_partition would emit, the static out shard elements and (if
// `max_tiles` is non-null) an upper bound of the number of `tile` x `tile` output tiles of those problems: whatever
// the buffers' row strides allow to be flattened, a flattened problem has no more tiles than its pieces.
int32_t count_partition(const gspmd_mesh* mesh, const DotRoles& roles,
                        const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                        const gspmd_sharding* out_sh, int64_t pid,
                        int64_t* n_problems, int64_t* out_static_elems, int64_t* max_tiles = nullptr, int tile = 256);

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace gspmd
