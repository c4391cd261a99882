// C-ABI entry points of libgspmd (see include/gspmd.h) and the kernel launchers.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <map>
#include <vector>

#include "../../include/gspmd.h"
#include "kernels_basic.h"
#include "kernels_mfma.h"
#include "plan.h"

using namespace gspmd;

namespace {

constexpr int64_t kWsAlign = 256;

// Workspace of gspmd_grouped_dot_noalloc: one copy per GPU the library is loaded on, held until the process ends.  In
// host code the array's name is only a handle: its device address is looked up once per device (scratch_address).
constexpr int64_t kScratchBytes = GSPMD_NOALLOC_MAX_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

void* scratch_address() {
  static std::once_flag once[kMaxDevices];
  static void* addr[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::call_once(once[dev], [dev] {
    void* p = nullptr;
    addr[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) == hipSuccess ? p : nullptr;
  });
  return addr[dev];
}

bool is_dtype(int32_t d) { return d == GSPMD_F32 || d == GSPMD_BF16; }

// A tensor with a zero-size dimension has no elements; its buffers may be null pointers.
bool has_no_elements(const gspmd_sharding* sh) {
  for (int i = 0; i < sh->rank; ++i) if (sh->global_shape[i] == 0) return true;
  return false;
}

int32_t check_buf(const gspmd_shard_buf* b) {
  if (!b) return GSPMD_ERR_NULL;
  if (!is_dtype(b->dtype)) return GSPMD_ERR_UNSUPPORTED;
  if (b->row_stride < 0) return GSPMD_ERR_BAD_BUFFER;
  return GSPMD_OK;
}

// Assign tile ids for tile edge (bm, bn) over the VALID extents; returns total tiles or -1 on overflow.
int64_t assign_tiles(std::vector<Problem>& ps, int bm, int bn) {
  int64_t t = 0;
  for (auto& p : ps) {
    const int64_t tm = (static_cast<int64_t>(p.Mv) + bm - 1) / bm, tn = (static_cast<int64_t>(p.Nv) + bn - 1) / bn;
    p.tile_begin = static_cast<int32_t>(t);
    p.tiles_n = static_cast<int32_t>(tn);
    t += tm * tn;
    if (t > INT32_MAX) return -1;
  }
  return t;
}

// Which contraction kernel a launch can take: the MFMA kernel with direct global->LDS loads needs 16-byte aligned
// operand pointers and leading dimensions that are multiples of 8 elements; its register-staged variant 4-byte aligned
// pointers and even leading dimensions; anything else (and fp32 operands) goes to the scalar-FMA kernel.
enum KernelPath { kPathFallback = 0, kPathMfmaStaged = 1, kPathMfmaDirect = 2 };

KernelPath kernel_path(const std::vector<Problem>& ps, int32_t in_dtype, int32_t layout, bool check_pointers = true) {
  if (in_dtype != GSPMD_BF16) return kPathFallback;
  // 32-bit byte offsets inside a tile: 256 rows of a K-contiguous operand, 32 of a K-major one
  const int32_t max_lda = (layout & GSPMD_LAYOUT_LHS_K_MAJOR) ? (1 << 24) : (1 << 22);
  const int32_t max_ldb = (layout & GSPMD_LAYOUT_RHS_K_CONTIGUOUS) ? (1 << 22) : (1 << 24);
  KernelPath path = kPathMfmaDirect;
  for (const auto& p : ps) {
    const uintptr_t ptrs = check_pointers ? reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B) : 0;
    if (p.lda > max_lda || p.ldb > max_ldb) return kPathFallback;
    if ((ptrs & 3) || ((p.lda | p.ldb) & 1)) return kPathFallback;
    if ((ptrs & 15) || ((p.lda | p.ldb) & 7)) path = kPathMfmaStaged;
  }
  return path;
}

bool mfma_eligible(const std::vector<Problem>& ps, int32_t in_dtype, int32_t layout) {
  return kernel_path(ps, in_dtype, layout) != kPathFallback;
}

// Run the contraction over all live tiles, then the zero fill of what the tiles do not cover.  Output tiles cover
// the valid extents only (rounded up to whole tiles, the kernel writes zeros inside a partly valid tile): tiles that
// would only write zeros are not interleaved with live ones, which would leave compute units idle (workgroups are
// placed in order), and cost no workgroup launches.  Tables of up to kInlineProblems problems and kInlineRects
// rectangles travel as kernel arguments; larger ones are uploaded into the workspace with a stream-ordered copy from
// a temporary host buffer (HIP stages a pageable source before the call returns).
// Where the MFMA kernel writes its per-workgroup timeline while gspmd_set_tile_timeline has one set (a profiling aid).
std::atomic<unsigned long long*> g_timeline{nullptr};
std::atomic<int> g_timeline_records{0};

// Workspace of a launch with joined problems: one arrival counter and join_count slots of kJoinSlotBytes per joined
// output tile.
constexpr int64_t kJoinSlotBytes = static_cast<int64_t>(kMfmaBM) * kMfmaBN * 4;
struct JoinSpace {
  uint32_t* counters = nullptr;
  float* partials = nullptr;
  int64_t tiles = 0;          // joined output tiles
};

constexpr int64_t kJoinSlack = int64_t(64) << 20;
// counters of `tiles` joined output tiles, then `slots` slots
int64_t joined_bytes(int64_t tiles, int64_t slots) { return round_up(tiles * 4, kWsAlign) + slots * kJoinSlotBytes; }

int64_t tiles_of(const Problem& p, int bm, int bn) {
  return ((static_cast<int64_t>(p.Mv) + bm - 1) / bm) * ((static_cast<int64_t>(p.Nv) + bn - 1) / bn);
}

int32_t launch_problems(std::vector<Problem>& all, int32_t layout, int32_t in_dtype, int32_t out_dtype, int32_t epilogue,
                        void* workspace, int64_t workspace_bytes, hipStream_t stream, const JoinSpace* join = nullptr) {
  // problems with an empty static output block write nothing
  all.erase(std::remove_if(all.begin(), all.end(), [](const Problem& p) { return p.Ms == 0 || p.Ns == 0; }), all.end());
  if (all.empty()) return GSPMD_OK;
  if (in_dtype == GSPMD_F32 && out_dtype != GSPMD_F32) return GSPMD_ERR_UNSUPPORTED;
  std::vector<Problem> ps;
  for (const auto& p : all) if (p.Mv > 0) ps.push_back(p);      // Mv, Nv, Kv are all zero or all positive
  const KernelPath path = kernel_path(ps, in_dtype, layout);
  const bool mfma = path != kPathFallback;
  if (join && !mfma) return GSPMD_ERR_UNSUPPORTED;              // the caller checks before it joins problems
  const int bm = mfma ? kMfmaBM : kGenTile, bn = mfma ? kMfmaBN : kGenTile;
  // Workgroups start in tile order and the launch ends when the last one does: problems whose tiles take longest
  // (the most K steps) go first, so that the compute units that are still busy at the end are busy with short tiles.
  if (!join)
    std::stable_sort(ps.begin(), ps.end(), [](const Problem& a, const Problem& b) { return a.Kv > b.Kv; });
  const int64_t tiles = assign_tiles(ps, bm, bn);
  if (tiles < 0) return GSPMD_ERR_UNSUPPORTED;
  std::vector<ZeroRect> rects;
  for (const auto& p : all) {
    if (p.join_slot > 0) continue;                              // one of the joined problems speaks for their common output
    // rows that the contraction kernel's tiles write or clear; the MFMA kernel's last tile row also clears up to
    // kRowsBelow rows below its footprint
    const int32_t rows_done = mfma ? rows_cleared(p.Mv, p.Ms)
                                   : static_cast<int32_t>(std::min<int64_t>(p.Ms, (static_cast<int64_t>(p.Mv) + bm - 1) / bm * bm));
    const int32_t cols_done = static_cast<int32_t>(std::min<int64_t>(p.Ns, (static_cast<int64_t>(p.Nv) + bn - 1) / bn * bn));
    if (rows_done < p.Ms) rects.push_back(ZeroRect{p.C, p.ldc, rows_done, p.Ms, 0, p.Ns, 0});
    if (cols_done < p.Ns && rows_done > 0) rects.push_back(ZeroRect{p.C, p.ldc, 0, rows_done, cols_done, p.Ns, 0});
  }
  const bool inline_tables = ps.size() <= static_cast<size_t>(kInlineProblems) && rects.size() <= static_cast<size_t>(kInlineRects);
  const int64_t prob_bytes = static_cast<int64_t>(ps.size()) * sizeof(Problem);
  const int64_t table_bytes = prob_bytes + static_cast<int64_t>(rects.size()) * sizeof(ZeroRect);
  // the workspace contract does not depend on which way the tables travel
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kWsAlign - 1)) || workspace_bytes < table_bytes)
    return GSPMD_ERR_WORKSPACE;
  const Problem* tab = nullptr;
  const ZeroRect* drects = nullptr;
  InlineProblems inl;
  InlineRects inl_rects;
  std::memset(&inl, 0, sizeof(inl));
  std::memset(&inl_rects, 0, sizeof(inl_rects));
  if (inline_tables) {
    if (!ps.empty()) std::memcpy(inl.p, ps.data(), static_cast<size_t>(prob_bytes));
    if (!rects.empty()) std::memcpy(inl_rects.r, rects.data(), rects.size() * sizeof(ZeroRect));
  } else {
    std::vector<char> host(static_cast<size_t>(table_bytes));
    if (prob_bytes) std::memcpy(host.data(), ps.data(), static_cast<size_t>(prob_bytes));
    if (!rects.empty()) std::memcpy(host.data() + prob_bytes, rects.data(), rects.size() * sizeof(ZeroRect));
    if (hipMemcpyAsync(workspace, host.data(), host.size(), hipMemcpyHostToDevice, stream) != hipSuccess)
      return GSPMD_ERR_DEVICE;
    tab = static_cast<const Problem*>(workspace);
    drects = reinterpret_cast<const ZeroRect*>(static_cast<const char*>(workspace) + prob_bytes);
  }
  const int n = static_cast<int>(ps.size());
  if (tiles > 0) {
    if (mfma) {
      if (join && join->tiles > 0) {
        const unsigned blocks = static_cast<unsigned>(std::min<int64_t>((join->tiles + 255) / 256, 1024));
        hipLaunchKernelGGL(zero_words_kernel, dim3(blocks), dim3(256), 0, stream, join->counters, join->tiles);
        if (hipGetLastError() != hipSuccess) return GSPMD_ERR_DEVICE;
      }
      if (!launch_dot_mfma(inl, tab, n, static_cast<int>(tiles), layout, out_dtype, path == kPathMfmaStaged, epilogue, join ? join->partials : nullptr,
                           join ? join->counters : nullptr, g_timeline.load(std::memory_order_acquire),
                           g_timeline_records.load(std::memory_order_acquire), stream)) return GSPMD_ERR_DEVICE;
    } else {
      const dim3 grid(static_cast<unsigned>(tiles)), block(256);
      if (in_dtype == GSPMD_F32)
        hipLaunchKernelGGL((dot_fallback_kernel<float, float>), grid, block, 0, stream, inl, tab, n, layout, epilogue);
      else if (out_dtype == GSPMD_F32)
        hipLaunchKernelGGL((dot_fallback_kernel<bf16_bits, float>), grid, block, 0, stream, inl, tab, n, layout, epilogue);
      else
        hipLaunchKernelGGL((dot_fallback_kernel<bf16_bits, bf16_bits>), grid, block, 0, stream, inl, tab, n, layout, epilogue);
      if (hipGetLastError() != hipSuccess) return GSPMD_ERR_DEVICE;
    }
  }
  if (!rects.empty()) {
    const int vec_elems = out_dtype == GSPMD_F32 ? 4 : 8;
    bool vec = true;
    int64_t most = 0;
    for (const auto& r : rects) {
      vec = vec && !(reinterpret_cast<uintptr_t>(r.C) & 15) && r.ldc % vec_elems == 0 && r.c0 % vec_elems == 0 &&
            (r.c1 - r.c0) % vec_elems == 0;
      most = std::max<int64_t>(most, static_cast<int64_t>(r.r1 - r.r0) * (r.c1 - r.c0));
    }
    const int64_t per_thread = vec ? vec_elems : 1;
    const unsigned gx = static_cast<unsigned>(std::min<int64_t>(std::max<int64_t>((most / per_thread + 255) / 256, 1), 2048));
    for (size_t first = 0; first < rects.size(); first += 65535) {       // grid.y is limited to 65535
      const unsigned gy = static_cast<unsigned>(std::min<size_t>(rects.size() - first, 65535));
      const dim3 grid(gx, gy), block(256);
      const ZeroRect* part = drects ? drects + first : nullptr;
      if (out_dtype == GSPMD_F32) {
        if (vec) hipLaunchKernelGGL((zero_rects_kernel<float, 4>), grid, block, 0, stream, inl_rects, part);
        else hipLaunchKernelGGL((zero_rects_kernel<float, 1>), grid, block, 0, stream, inl_rects, part);
      } else {
        if (vec) hipLaunchKernelGGL((zero_rects_kernel<bf16_bits, 8>), grid, block, 0, stream, inl_rects, part);
        else hipLaunchKernelGGL((zero_rects_kernel<bf16_bits, 1>), grid, block, 0, stream, inl_rects, part);
      }
    }
    if (hipGetLastError() != hipSuccess) return GSPMD_ERR_DEVICE;
  }
  return GSPMD_OK;
}

int32_t launch_reduce(const float* const* partials, int n_partials, int64_t rows, int64_t cols, int64_t ld_in,
                      void* out, int64_t ld_out, int32_t out_dtype, hipStream_t stream) {
  if (rows == 0 || cols == 0) return GSPMD_OK;
  PartialPtrs pp;
  uintptr_t bits = reinterpret_cast<uintptr_t>(out);
  for (int i = 0; i < kMaxPartials; ++i) pp.p[i] = nullptr;
  for (int i = 0; i < n_partials; ++i) { pp.p[i] = partials[i]; bits |= reinterpret_cast<uintptr_t>(partials[i]); }
  const bool vec = !(bits & 15) && !(cols & 3) && !(ld_in & 3) && !(ld_out & 3);
  const int64_t work = rows * (vec ? cols / 4 : cols);
  const unsigned blocks = static_cast<unsigned>(std::min<int64_t>((work + 255) / 256, 1 << 20));   // one vector per thread up to 1 GiB of fp32
  const dim3 grid(blocks), block(256);
  if (out_dtype == GSPMD_F32) {
    if (vec) hipLaunchKernelGGL((reduce_partials_kernel<float, 4>), grid, block, 0, stream, pp, n_partials, rows, cols, ld_in, static_cast<float*>(out), ld_out);
    else hipLaunchKernelGGL((reduce_partials_kernel<float, 1>), grid, block, 0, stream, pp, n_partials, rows, cols, ld_in, static_cast<float*>(out), ld_out);
  } else {
    if (vec) hipLaunchKernelGGL((reduce_partials_kernel<bf16_bits, 4>), grid, block, 0, stream, pp, n_partials, rows, cols, ld_in, static_cast<bf16_bits*>(out), ld_out);
    else hipLaunchKernelGGL((reduce_partials_kernel<bf16_bits, 1>), grid, block, 0, stream, pp, n_partials, rows, cols, ld_in, static_cast<bf16_bits*>(out), ld_out);
  }
  return hipGetLastError() == hipSuccess ? GSPMD_OK : GSPMD_ERR_DEVICE;
}

bool is_contracting(int32_t c) { return c == GSPMD_AXIS_CONTRACTING || c == GSPMD_AXIS_CONTRACTING_SCATTER; }

bool has_contracting(const gspmd_mesh* mesh, const int32_t* cls) {
  for (int a = 0; a < mesh->rank; ++a) if (is_contracting(cls[a])) return true;
  return false;
}

bool has_scatter(const gspmd_mesh* mesh, const int32_t* cls) {
  for (int a = 0; a < mesh->rank; ++a) if (cls[a] == GSPMD_AXIS_CONTRACTING_SCATTER) return true;
  return false;
}

bool is_epilogue(int32_t e) { return e == GSPMD_EPILOGUE_NONE || e == GSPMD_EPILOGUE_RELU; }

// The sharding of a partition's partial sum: the out sharding with the dimensions that a scatter mesh dimension
// splits made whole again (the slice is taken after the sum).
void partial_mapping(const gspmd_mesh* mesh, const int32_t* cls, const gspmd_sharding* out_sh, int32_t* map) {
  for (int i = 0; i < out_sh->rank; ++i) {
    const int a = out_sh->dims_mapping[i];
    map[i] = (a >= 0 && a < mesh->rank && cls[a] == GSPMD_AXIS_CONTRACTING_SCATTER) ? -1 : a;
  }
}

// out shard of partition `pid` = epilogue(sum of the group's partials) restricted to the shard's place in them.
int32_t launch_reduce_scatter(const gspmd_mesh* mesh, const gspmd_sharding* out_sh, const gspmd_sharding* part_sh, int64_t pid,
                              const float* const* partials, int n_partials, const gspmd_shard_buf* out, int32_t epilogue,
                              hipStream_t stream) {
  Bounds ob, pb;
  int32_t st;
  if ((st = shard_bounds(mesh, out_sh, pid, &ob)) != GSPMD_OK) return st;
  if ((st = shard_bounds(mesh, part_sh, pid, &pb)) != GSPMD_OK) return st;
  ScatterDesc d;
  std::memset(&d, 0, sizeof(d));
  const int r = ob.rank, last = r - 1;
  d.rank = r;
  int64_t rows = 1, in_stride = 1;
  for (int i = last; i >= 0; --i) {
    if (ob.shard[i] > INT32_MAX) return GSPMD_ERR_UNSUPPORTED;
    d.shard[i] = static_cast<int32_t>(ob.shard[i]);
    d.valid[i] = static_cast<int32_t>(ob.valid[i]);
    d.in_off[i] = ob.offset[i] - pb.offset[i];
    d.in_stride[i] = in_stride;
    in_stride *= pb.shard[i];
    if (i < last) rows *= ob.shard[i];
  }
  if (rows > INT32_MAX) return GSPMD_ERR_UNSUPPORTED;
  d.rows = static_cast<int32_t>(rows);
  d.out_stride[last] = 1;
  if (r >= 2) {
    const int64_t rs = out->row_stride > 0 ? out->row_stride : ob.shard[last];
    if (rs < ob.shard[last]) return GSPMD_ERR_BAD_BUFFER;
    d.out_stride[r - 2] = rs;
    for (int i = r - 3; i >= 0; --i) d.out_stride[i] = d.out_stride[i + 1] * ob.shard[i + 1];
  }
  if (rows == 0 || ob.shard[last] == 0) return GSPMD_OK;
  PartialPtrs pp;
  uintptr_t bits = reinterpret_cast<uintptr_t>(out->data);
  for (int i = 0; i < kMaxPartials; ++i) pp.p[i] = nullptr;
  for (int i = 0; i < n_partials; ++i) { pp.p[i] = partials[i]; bits |= reinterpret_cast<uintptr_t>(partials[i]); }
  bool vec = !(bits & 15) && !(ob.shard[last] & 3) && !(pb.shard[last] & 3) && !(d.in_off[last] & 3);
  for (int i = 0; i < last; ++i) vec = vec && !(d.in_stride[i] & 3) && !(d.out_stride[i] & 3);
  const int64_t cols_v = (ob.shard[last] + (vec ? 3 : 0)) / (vec ? 4 : 1);
  // one vector per thread (a workgroup per 256 vectors of a row) up to the grid limit, beyond that each thread walks
  // down its column: measured faster than fewer workgroups with a loop (6.2 against 5.4 TB/s on 2.4 GB)
  const int64_t gx = (cols_v + 255) / 256;
  const dim3 block(256), grid(static_cast<unsigned>(gx), static_cast<unsigned>(std::min<int64_t>(rows, 65535)));
  if (out->dtype == GSPMD_F32) {
    if (vec) hipLaunchKernelGGL((reduce_scatter_kernel<float, 4>), grid, block, 0, stream, d, pp, n_partials, static_cast<float*>(out->data), epilogue);
    else hipLaunchKernelGGL((reduce_scatter_kernel<float, 1>), grid, block, 0, stream, d, pp, n_partials, static_cast<float*>(out->data), epilogue);
  } else {
    if (vec) hipLaunchKernelGGL((reduce_scatter_kernel<bf16_bits, 4>), grid, block, 0, stream, d, pp, n_partials, static_cast<bf16_bits*>(out->data), epilogue);
    else hipLaunchKernelGGL((reduce_scatter_kernel<bf16_bits, 1>), grid, block, 0, stream, d, pp, n_partials, static_cast<bf16_bits*>(out->data), epilogue);
  }
  return hipGetLastError() == hipSuccess ? GSPMD_OK : GSPMD_ERR_DEVICE;
}

}  // namespace

extern "C" {

const char* gspmd_status_string(int32_t s) {
  switch (s) {
    case GSPMD_OK: return "ok";
    case GSPMD_ERR_NULL: return "null pointer";
    case GSPMD_ERR_BAD_MESH: return "bad device mesh";
    case GSPMD_ERR_BAD_SHARDING: return "bad sharding";
    case GSPMD_ERR_PARTITION_RANGE: return "partition id out of range";
    case GSPMD_ERR_BAD_DOT_DIMS: return "bad dot dimension numbers";
    case GSPMD_ERR_NEEDS_RESHARD: return "shardings need resharding";
    case GSPMD_ERR_UNSUPPORTED: return "unsupported dtype or layout";
    case GSPMD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GSPMD_ERR_DEVICE: return "HIP error";
    case GSPMD_ERR_BAD_BUFFER: return "bad shard buffer";
    case GSPMD_ERR_HOST_MEMORY: return "host allocation failed";
    default: return "unknown status";
  }
}

int32_t gspmd_shard_bounds(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid,
                           int64_t* offset, int64_t* valid_len, int64_t* shard_size) try {
  if (!offset || !valid_len) return GSPMD_ERR_NULL;
  int32_t st = validate_mesh(mesh, nullptr);
  if (st != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, sh)) != GSPMD_OK) return st;
  Bounds b;
  if ((st = shard_bounds(mesh, sh, pid, &b)) != GSPMD_OK) return st;
  for (int i = 0; i < b.rank; ++i) {
    offset[i] = b.offset[i];
    valid_len[i] = b.valid[i];
    if (shard_size) shard_size[i] = b.shard[i];
  }
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_classify_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                           const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                           const gspmd_sharding* out_sh, int32_t* axis_class) try {
  if (!axis_class) return GSPMD_ERR_NULL;
  DotRoles r;
  int32_t cls[kMaxRank];
  const int32_t st = analyse_dot(mesh, dims, lhs_sh, rhs_sh, out_sh, &r, cls);
  if (st != GSPMD_OK) return st;
  for (int a = 0; a < mesh->rank; ++a) axis_class[a] = cls[a];
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_infer_out_sharding(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                 const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                 int32_t* out_mapping, int64_t* out_shape, int32_t* out_rank) try {
  if (!out_mapping || !dims) return GSPMD_ERR_NULL;
  int32_t st = validate_mesh(mesh, nullptr);
  if (st != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, lhs_sh)) != GSPMD_OK || (st = validate_sharding(mesh, rhs_sh)) != GSPMD_OK) return st;
  // a provisional, unsplit output lets analyse_dot check the dimension numbers and name the roles
  const int nb = dims->n_batch, nc = dims->n_contract;
  if (nb < 0 || nc < 0 || nb + nc > lhs_sh->rank || nb + nc > rhs_sh->rank) return GSPMD_ERR_BAD_DOT_DIMS;
  const int rank = lhs_sh->rank + rhs_sh->rank - nb - 2 * nc;
  if (rank <= 0 || rank > kMaxRank) return GSPMD_ERR_UNSUPPORTED;
  int64_t shape[kMaxRank];
  int32_t map[kMaxRank];
  std::vector<bool> lused(static_cast<size_t>(lhs_sh->rank), false), rused(static_cast<size_t>(rhs_sh->rank), false);
  for (int i = 0; i < nb; ++i) {
    const int a = dims->lhs_batch ? dims->lhs_batch[i] : -1, b = dims->rhs_batch ? dims->rhs_batch[i] : -1;
    if (a < 0 || a >= lhs_sh->rank || b < 0 || b >= rhs_sh->rank) return GSPMD_ERR_BAD_DOT_DIMS;
    lused[static_cast<size_t>(a)] = rused[static_cast<size_t>(b)] = true;
  }
  for (int i = 0; i < nc; ++i) {
    const int a = dims->lhs_contract ? dims->lhs_contract[i] : -1, b = dims->rhs_contract ? dims->rhs_contract[i] : -1;
    if (a < 0 || a >= lhs_sh->rank || b < 0 || b >= rhs_sh->rank) return GSPMD_ERR_BAD_DOT_DIMS;
    lused[static_cast<size_t>(a)] = rused[static_cast<size_t>(b)] = true;
  }
  int n = 0;
  for (int i = 0; i < nb; ++i) { shape[n] = lhs_sh->global_shape[dims->lhs_batch[i]]; map[n++] = -1; }
  for (int i = 0; i < lhs_sh->rank; ++i) if (!lused[static_cast<size_t>(i)]) { shape[n] = lhs_sh->global_shape[i]; map[n++] = -1; }
  for (int i = 0; i < rhs_sh->rank; ++i) if (!rused[static_cast<size_t>(i)]) { shape[n] = rhs_sh->global_shape[i]; map[n++] = -1; }
  if (n != rank) return GSPMD_ERR_BAD_DOT_DIMS;
  gspmd_sharding out{rank, shape, map};
  DotRoles r;
  // roles and size checks only: run the analysis on a 1-partition mesh so that no pattern is rejected yet
  const int64_t one = 1, zero = 0;
  gspmd_mesh unit{1, &one, &zero};
  std::vector<int32_t> lm(static_cast<size_t>(lhs_sh->rank), -1), rm(static_cast<size_t>(rhs_sh->rank), -1);
  gspmd_sharding l1{lhs_sh->rank, lhs_sh->global_shape, lm.data()}, r1{rhs_sh->rank, rhs_sh->global_shape, rm.data()};
  if ((st = analyse_dot(&unit, dims, &l1, &r1, &out, &r, nullptr)) != GSPMD_OK) return st;
  for (int a = 0; a < mesh->rank; ++a) {
    if (mesh->shape[a] == 1) continue;                // splits nothing
    int ld = -1, rd = -1;
    for (int i = 0; i < lhs_sh->rank; ++i) if (lhs_sh->dims_mapping[i] == a) ld = i;
    for (int i = 0; i < rhs_sh->rank; ++i) if (rhs_sh->dims_mapping[i] == a) rd = i;
    if (ld < 0 && rd < 0) continue;
    auto idx = [](const int* list, int cnt, int v) { for (int i = 0; i < cnt; ++i) if (list[i] == v) return i; return -1; };
    const int lb = ld >= 0 ? idx(r.lhs_batch, r.nb, ld) : -1, rbb = rd >= 0 ? idx(r.rhs_batch, r.nb, rd) : -1;
    const int lcn = ld >= 0 ? idx(r.lhs_contract, r.nc, ld) : -1, rcn = rd >= 0 ? idx(r.rhs_contract, r.nc, rd) : -1;
    const int lf = ld >= 0 ? idx(r.lhs_free, r.nlf, ld) : -1, rf = rd >= 0 ? idx(r.rhs_free, r.nrf, rd) : -1;
    if (lb >= 0 || rbb >= 0) {                        // a batch pair must be split alike on both sides
      if (lb < 0 || rbb != lb) return GSPMD_ERR_NEEDS_RESHARD;
      map[lb] = a;
    } else if (lcn >= 0 || rcn >= 0) {                // so must a contracting pair; the output is a partial sum
      if (lcn < 0 || rcn != lcn) return GSPMD_ERR_NEEDS_RESHARD;
    } else if (lf >= 0 && rf >= 0) {                  // one mesh dimension cannot split two output dimensions
      return GSPMD_ERR_NEEDS_RESHARD;
    } else if (lf >= 0) {
      map[r.nb + lf] = a;
    } else {
      map[r.nb + r.nlf + rf] = a;
    }
  }
  for (int i = 0; i < rank; ++i) { out_mapping[i] = map[i]; if (out_shape) out_shape[i] = shape[i]; }
  if (out_rank) *out_rank = rank;
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_plan_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                       const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh, const gspmd_sharding* out_sh,
                       int64_t lhs_row_stride, int64_t rhs_row_stride, int64_t out_row_stride,
                       int64_t pid, const int64_t* lhs_fill,
                       gspmd_gemm_desc* descs, int64_t capacity, int64_t* count) try {
  if (!count || (capacity > 0 && !descs)) return GSPMD_ERR_NULL;
  if (capacity < 0 || lhs_row_stride < 0 || rhs_row_stride < 0 || out_row_stride < 0) return GSPMD_ERR_BAD_BUFFER;
  DotRoles r;
  int32_t cls[kMaxRank];
  int32_t st = analyse_dot(mesh, dims, lhs_sh, rhs_sh, out_sh, &r, cls);
  if (st != GSPMD_OK) return st;
  // plan against made-up base addresses far apart, with 1-byte elements, so that pointer differences are element offsets
  const uintptr_t base_a = uintptr_t(1) << 44, base_b = uintptr_t(2) << 44, base_c = uintptr_t(3) << 44;
  gspmd_shard_buf la{reinterpret_cast<void*>(base_a), GSPMD_F32, lhs_row_stride};
  gspmd_shard_buf rb{reinterpret_cast<void*>(base_b), GSPMD_F32, rhs_row_stride};
  gspmd_shard_buf oc{reinterpret_cast<void*>(base_c), GSPMD_F32, out_row_stride};
  std::vector<Problem> ps;
  int64_t elems = 0;
  int32_t layout = 0;
  if ((st = plan_partition(mesh, r, &la, lhs_sh, &rb, rhs_sh, &oc, out_sh, pid, lhs_fill, nullptr, &ps, &elems, &layout)) != GSPMD_OK) return st;
  *count = static_cast<int64_t>(ps.size());
  // the operand addresses here are made up: the path is named from the leading dimensions alone
  std::vector<Problem> live;
  for (const auto& p : ps) if (p.Mv > 0) live.push_back(p);
  const KernelPath kp = kernel_path(live, GSPMD_BF16, layout, false);
  const int32_t path = kp == kPathMfmaDirect ? GSPMD_KERNEL_MFMA : kp == kPathMfmaStaged ? GSPMD_KERNEL_MFMA_STAGED : GSPMD_KERNEL_SCALAR;
  for (int64_t i = 0; i < std::min<int64_t>(capacity, *count); ++i) {
    const Problem& p = ps[static_cast<size_t>(i)];
    gspmd_gemm_desc& d = descs[i];
    d.a_offset = static_cast<int64_t>(reinterpret_cast<uintptr_t>(p.A) - base_a) / 4;
    d.b_offset = static_cast<int64_t>(reinterpret_cast<uintptr_t>(p.B) - base_b) / 4;
    d.c_offset = static_cast<int64_t>(reinterpret_cast<uintptr_t>(p.C) - base_c) / 4;
    d.lda = p.lda; d.ldb = p.ldb; d.ldc = p.ldc;
    d.m_valid = p.Mv; d.n_valid = p.Nv; d.k_valid = p.Kv;
    d.m_static = p.Ms; d.n_static = p.Ns;
    d.layout = layout;
    d.kernel = path;
    d.reserved = 0;
  }
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_dot_workspace_bytes(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                  const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                  const gspmd_sharding* out_sh, int64_t pid, int32_t /*has_fill*/,
                                  int64_t* bytes) try {
  if (!bytes) return GSPMD_ERR_NULL;
  DotRoles r;
  int32_t cls[kMaxRank];
  int32_t st = analyse_dot(mesh, dims, lhs_sh, rhs_sh, out_sh, &r, cls);
  if (st != GSPMD_OK) return st;
  int64_t P = 1;
  for (int a = 0; a < mesh->rank; ++a) P *= mesh->shape[a];
  if (pid < -1 || pid >= P) return GSPMD_ERR_PARTITION_RANGE;
  int64_t n_prob = 0, partial_bytes = 0, tiles = 0;
  const bool contracting = has_contracting(mesh, cls);
  int32_t pmap[kMaxRank];
  partial_mapping(mesh, cls, out_sh, pmap);
  const gspmd_sharding part_sh{out_sh->rank, out_sh->global_shape, pmap};
  for (int64_t p = (pid < 0 ? 0 : pid); p < (pid < 0 ? P : pid + 1); ++p) {
    int64_t n, e, t;
    if ((st = count_partition(mesh, r, lhs_sh, rhs_sh, &part_sh, p, &n, &e, &t, kMfmaBM)) != GSPMD_OK) return st;
    n_prob += n;
    tiles = std::min<int64_t>(tiles + t, int64_t(1) << 40);
    if (pid < 0 && contracting) partial_bytes += round_up(e * 4, kWsAlign);
  }
  // A grouped call with a contracting mesh dimension keeps its partial sums either as one dense fp32 array per
  // partition or, when the problems can be joined in one launch, as one slot per output tile and partition plus a
  // counter per tile; the second layout is offered only while it stays within reach of the first.
  if (pid < 0 && contracting) {
    const int64_t joined = joined_bytes(tiles, tiles);
    if (joined <= 2 * partial_bytes + kJoinSlack) partial_bytes = std::max(partial_bytes, joined);
  }
  *bytes = round_up(std::max<int64_t>(n_prob, 1) * kTableBytesPerProblem, kWsAlign) + partial_bytes;
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_local_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                        const gspmd_shard_buf* lhs, const gspmd_sharding* lhs_sh,
                        const gspmd_shard_buf* rhs, const gspmd_sharding* rhs_sh,
                        const gspmd_shard_buf* out, const gspmd_sharding* out_sh,
                        int64_t pid, const int64_t* lhs_fill, int32_t epilogue,
                        void* workspace, int64_t workspace_bytes, void* hip_stream) try {
  int32_t st;
  if (!is_epilogue(epilogue)) return GSPMD_ERR_UNSUPPORTED;
  if ((st = check_buf(lhs)) != GSPMD_OK || (st = check_buf(rhs)) != GSPMD_OK || (st = check_buf(out)) != GSPMD_OK) return st;
  DotRoles r;
  int32_t cls[kMaxRank];
  if ((st = analyse_dot(mesh, dims, lhs_sh, rhs_sh, out_sh, &r, cls)) != GSPMD_OK) return st;
  if (lhs->dtype != rhs->dtype) return GSPMD_ERR_UNSUPPORTED;
  if (has_contracting(mesh, cls) && (out->dtype != GSPMD_F32 || epilogue != GSPMD_EPILOGUE_NONE)) return GSPMD_ERR_UNSUPPORTED;
  if (has_scatter(mesh, cls)) return GSPMD_ERR_UNSUPPORTED;   // a slice of a sum exists only after the exchange
  std::vector<Problem> ps;
  int64_t elems = 0;
  int32_t layout = 0;
  if ((st = plan_partition(mesh, r, lhs, lhs_sh, rhs, rhs_sh, out, out_sh, pid, lhs_fill, nullptr, &ps, &elems, &layout)) != GSPMD_OK)
    return st;
  for (const auto& p : ps)
    if ((p.Kv && (!p.A || !p.B)) || !p.C) return GSPMD_ERR_NULL;
  return launch_problems(ps, layout, lhs->dtype, out->dtype, epilogue, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_grouped_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                          const gspmd_shard_buf* lhs_shards, const gspmd_sharding* lhs_sh,
                          const gspmd_shard_buf* rhs_shards, const gspmd_sharding* rhs_sh,
                          const gspmd_shard_buf* out_shards, const gspmd_sharding* out_sh,
                          const int64_t* lhs_fill, int32_t epilogue,
                          void* workspace, int64_t workspace_bytes, void* hip_stream) try {
  if (!lhs_shards || !rhs_shards || !out_shards) return GSPMD_ERR_NULL;
  if (!is_epilogue(epilogue)) return GSPMD_ERR_UNSUPPORTED;
  DotRoles r;
  int32_t cls[kMaxRank];
  int32_t st;
  if ((st = analyse_dot(mesh, dims, lhs_sh, rhs_sh, out_sh, &r, cls)) != GSPMD_OK) return st;
  int64_t P = 1;
  for (int a = 0; a < mesh->rank; ++a) P *= mesh->shape[a];
  const int32_t in_dtype = lhs_shards[0].dtype, out_dtype = out_shards[0].dtype;
  for (int64_t p = 0; p < P; ++p) {
    if ((st = check_buf(&lhs_shards[p])) != GSPMD_OK || (st = check_buf(&rhs_shards[p])) != GSPMD_OK ||
        (st = check_buf(&out_shards[p])) != GSPMD_OK) return st;
    if (lhs_shards[p].dtype != in_dtype || rhs_shards[p].dtype != in_dtype || out_shards[p].dtype != out_dtype)
      return GSPMD_ERR_UNSUPPORTED;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const bool contracting = has_contracting(mesh, cls);

  // workspace = [problem table][fp32 partial of partition 0][partial of partition 1]...
  int64_t need = 0;
  if ((st = gspmd_dot_workspace_bytes(mesh, dims, lhs_sh, rhs_sh, out_sh, -1, lhs_fill != nullptr, &need)) != GSPMD_OK) return st;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kWsAlign - 1)) || workspace_bytes < need) return GSPMD_ERR_WORKSPACE;
  int64_t n_bound = 0;
  std::vector<int64_t> elems(static_cast<size_t>(P), 0);
  int32_t pmap[kMaxRank];
  partial_mapping(mesh, cls, out_sh, pmap);
  const gspmd_sharding part_sh{out_sh->rank, out_sh->global_shape, pmap};   // == out_sh unless a sum is scattered
  for (int64_t p = 0; p < P; ++p) {
    int64_t n;
    if ((st = count_partition(mesh, r, lhs_sh, rhs_sh, &part_sh, p, &n, &elems[static_cast<size_t>(p)])) != GSPMD_OK) return st;
    n_bound += n;
  }
  char* partial_base = static_cast<char*>(workspace) + round_up(std::max<int64_t>(n_bound, 1) * kTableBytesPerProblem, kWsAlign);
  std::vector<float*> partial(static_cast<size_t>(P), nullptr);
  if (contracting) {
    int64_t off = 0;
    for (int64_t p = 0; p < P; ++p) {
      partial[static_cast<size_t>(p)] = reinterpret_cast<float*>(partial_base + off);
      off += round_up(elems[static_cast<size_t>(p)] * 4, kWsAlign);
    }
  }

  // Reduce groups: partitions that differ only along contracting mesh dimensions, in ascending mesh position.
  std::map<std::vector<int64_t>, std::vector<std::pair<int64_t, int64_t>>> groups;   // key -> (lin pos, pid)
  if (contracting) {
    for (int64_t p = 0; p < P; ++p) {
      int64_t coords[kMaxRank];
      if ((st = mesh_coords(mesh, p, coords)) != GSPMD_OK) return st;
      std::vector<int64_t> key;
      int64_t pos = 0;
      for (int a = 0; a < mesh->rank; ++a) {
        if (is_contracting(cls[a])) pos = pos * mesh->shape[a] + coords[a];
        else key.push_back(coords[a]);
      }
      groups[key].emplace_back(pos, p);
    }
    for (auto& kv : groups) std::sort(kv.second.begin(), kv.second.end());
  }

  // One launch for the whole sum (the AllReduce / ReduceScatter of Section 4.2 folded into the contraction): the
  // problems of a reduce group's members are joined -- every output tile gets one contribution per member, added in
  // ascending mesh position by whichever workgroup finishes last.  Two shapes qualify.  AllReduce: every member writes
  // the same out buffer and lowers to the same output blocks.  ReduceScatter along the output's last dimension, when
  // that is the only non-contracting rhs dimension and the scatter mesh dimension the only contracting one: each
  // member's problems are cut into the column ranges the members own, and the pieces for one owner are joined into that
  // owner's out shard.  Otherwise (other scattered sums, members with out buffers of their own, operands the MFMA
  // kernel cannot take, a workspace sized for the dense layout only) the partials go to dense arrays and a second
  // kernel sums them.
  int n_contracting_dims = 0;
  for (int a = 0; a < mesh->rank; ++a) n_contracting_dims += is_contracting(cls[a]) ? 1 : 0;
  const int last_out = out_sh->rank - 1;
  const bool scatter = has_scatter(mesh, cls);
  const bool scatter_by_columns = scatter && n_contracting_dims == 1 && r.nrf == 1 && out_sh->dims_mapping[last_out] >= 0 &&
                                  cls[out_sh->dims_mapping[last_out]] == GSPMD_AXIS_CONTRACTING_SCATTER;
  if (contracting && (!scatter || scatter_by_columns) && in_dtype == GSPMD_BF16) {
    std::vector<Problem> joined;
    int32_t jlayout = 0;
    int64_t jtiles = 0, jslots = 0;
    bool ok = true;
    const size_t out_esize = out_dtype == GSPMD_BF16 ? 2 : 4;
    char* const dummy_c = reinterpret_cast<char*>(uintptr_t(1) << 44);      // never dereferenced: offsets are read off it
    for (auto& kv : groups) {
      const auto& members = kv.second;
      // the members' problems: against the shared out buffer, or (scattered) against a made-up dense partial
      std::vector<std::vector<Problem>> base(members.size());
      const gspmd_shard_buf& o0 = out_shards[members[0].second];
      for (size_t m = 0; m < members.size() && ok; ++m) {
        const int64_t p = members[m].second;
        if (!scatter) ok = out_shards[p].data == o0.data && out_shards[p].row_stride == o0.row_stride;
        if (!ok) break;
        int64_t e = 0;
        if ((st = plan_partition(mesh, r, &lhs_shards[p], lhs_sh, &rhs_shards[p], rhs_sh, &out_shards[p], scatter ? &part_sh : out_sh, p,
                                 lhs_fill, scatter ? dummy_c : nullptr, &base[m], &e, &jlayout)) != GSPMD_OK) return st;
        for (const auto& q : base[m])
          if ((q.Kv && (!q.A || !q.B)) || !q.C) return GSPMD_ERR_NULL;
        ok = base[m].size() == base[0].size();
      }
      if (!ok) break;
      // one round per owner of output columns: the one shared buffer, or every member's own slice
      for (size_t owner = 0; ok && owner < (scatter ? members.size() : 1); ++owner) {
        std::vector<std::vector<Problem>> pm = base;
        if (scatter) {
          const int64_t po = members[owner].second;
          Bounds ob;
          if ((st = shard_bounds(mesh, out_sh, po, &ob)) != GSPMD_OK) return st;
          if (!out_shards[po].data && ob.shard[last_out] > 0) return GSPMD_ERR_NULL;
          const int64_t off = ob.offset[last_out], width = ob.shard[last_out];
          const int64_t ldo = out_sh->rank >= 2 && out_shards[po].row_stride > 0 ? out_shards[po].row_stride : width;
          if (ldo < width || ldo > INT32_MAX || width > INT32_MAX) { ok = false; break; }
          for (auto& list : pm)
            for (auto& q : list) {
              const int64_t elem = (static_cast<char*>(q.C) - dummy_c) / 4;          // offset inside the dense partial
              if (q.Ns <= 0 || elem % q.Ns != 0) { ok = false; break; }
              const int64_t row = elem / q.Ns;
              const int64_t nv = std::max<int64_t>(0, std::min<int64_t>(ob.valid[last_out], static_cast<int64_t>(q.Nv) - off));
              const int64_t b_step = (jlayout & GSPMD_LAYOUT_RHS_K_CONTIGUOUS) ? off * q.ldb : off;
              q.B = static_cast<const char*>(q.B) + b_step * 2;
              q.C = static_cast<char*>(out_shards[po].data) + row * ldo * static_cast<int64_t>(out_esize);
              q.ldc = static_cast<int32_t>(ldo);
              q.Ns = static_cast<int32_t>(width);
              q.Nv = static_cast<int32_t>(nv);
              if (q.Mv == 0 || q.Nv == 0 || q.Kv == 0) q.Mv = q.Nv = q.Kv = 0;
            }
        }
        for (size_t i = 0; ok && i < pm[0].size(); ++i) {
          std::vector<size_t> live;
          for (size_t m = 0; m < members.size(); ++m) {
            const Problem &q = pm[m][i], &q0 = pm[0][i];
            ok = ok && q.C == q0.C && q.ldc == q0.ldc && q.Ms == q0.Ms && q.Ns == q0.Ns;
            if (q.Kv > 0) {
              if (!live.empty()) ok = ok && q.Mv == pm[live[0]][i].Mv && q.Nv == pm[live[0]][i].Nv;
              live.push_back(m);
            }
          }
          if (!ok || live.size() > static_cast<size_t>(kMaxPartials)) { ok = false; break; }
          if (live.size() <= 1) {
            joined.push_back(pm[live.empty() ? 0 : live[0]][i]);       // nothing to add up (a dead problem still has its zero fill)
            continue;
          }
          const int64_t t = tiles_of(pm[live[0]][i], kMfmaBM, kMfmaBN);
          for (size_t k = 0; k < live.size(); ++k) {
            Problem q = pm[live[k]][i];
            q.join_count = static_cast<int32_t>(live.size());
            q.join_slot = static_cast<int32_t>(k);
            q.join_first = static_cast<int32_t>(jtiles);
            joined.push_back(q);
          }
          jtiles += t;
          jslots += t * static_cast<int64_t>(live.size());
          if (jtiles > INT32_MAX) { ok = false; break; }
        }
      }
      if (!ok) break;
    }
    if (ok) {
      std::vector<Problem> live;
      for (const auto& q : joined) if (q.Mv > 0) live.push_back(q);
      ok = mfma_eligible(live, in_dtype, jlayout);
    }
    const int64_t table_area = partial_base - static_cast<char*>(workspace);
    if (ok && table_area + joined_bytes(jtiles, jslots) <= workspace_bytes) {
      JoinSpace js;
      js.counters = reinterpret_cast<uint32_t*>(partial_base);
      js.partials = reinterpret_cast<float*>(partial_base + round_up(jtiles * 4, kWsAlign));
      js.tiles = jtiles;
      return launch_problems(joined, jlayout, in_dtype, out_dtype, epilogue, workspace, workspace_bytes, stream, &js);
    }
  }

  std::vector<Problem> ps;
  // Partitions that hold the same operands and write the same buffer (replicas along an
  // unused mesh dimension) need the product only once.
  std::map<std::array<const void*, 3>, int64_t> done;
  int32_t layout = 0;
  for (int64_t p = 0; p < P; ++p) {
    if (!contracting) {
      std::array<const void*, 3> key = {lhs_shards[p].data, rhs_shards[p].data, out_shards[p].data};
      if (done.count(key)) continue;
      done[key] = p;
    }
    int64_t e = 0;
    const size_t before = ps.size();
    st = plan_partition(mesh, r, &lhs_shards[p], lhs_sh, &rhs_shards[p], rhs_sh, &out_shards[p], &part_sh, p, lhs_fill,
                        contracting ? partial[static_cast<size_t>(p)] : nullptr, &ps, &e, &layout);
    if (st != GSPMD_OK) return st;
    for (size_t i = before; i < ps.size(); ++i)
      if ((ps[i].Kv && (!ps[i].A || !ps[i].B)) || !ps[i].C) return GSPMD_ERR_NULL;
  }
  st = launch_problems(ps, layout, in_dtype, contracting ? GSPMD_F32 : out_dtype, contracting ? GSPMD_EPILOGUE_NONE : epilogue,
                       workspace, workspace_bytes, stream);
  if (st != GSPMD_OK || !contracting) return st;

  // Sum the partials of each reduce group, ascending in mesh position, into every distinct out buffer of the group.
  for (auto& kv : groups) {
    auto& members = kv.second;
    if (members.size() > static_cast<size_t>(kMaxPartials)) return GSPMD_ERR_UNSUPPORTED;
    std::vector<const float*> ptrs;
    for (auto& m : members) ptrs.push_back(partial[static_cast<size_t>(m.second)]);
    std::vector<void*> written;
    for (auto& m : members) {
      const gspmd_shard_buf& o = out_shards[m.second];
      if (std::find(written.begin(), written.end(), o.data) != written.end()) continue;
      written.push_back(o.data);
      if ((st = launch_reduce_scatter(mesh, out_sh, &part_sh, m.second, ptrs.data(), static_cast<int>(ptrs.size()), &o, epilogue,
                                      stream)) != GSPMD_OK)
        return st;
    }
  }
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_grouped_dot_noalloc(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                  const gspmd_shard_buf* lhs_shards, const gspmd_sharding* lhs_sh,
                                  const gspmd_shard_buf* rhs_shards, const gspmd_sharding* rhs_sh,
                                  const gspmd_shard_buf* out_shards, const gspmd_sharding* out_sh,
                                  const int64_t* lhs_fill, int32_t epilogue, void* hip_stream) try {
  int64_t need = 0;
  const int32_t st = gspmd_dot_workspace_bytes(mesh, dims, lhs_sh, rhs_sh, out_sh, -1, lhs_fill != nullptr, &need);
  if (st != GSPMD_OK) return st;
  if (need > kScratchBytes) return GSPMD_ERR_WORKSPACE;     // launch tables + fp32 partials do not fit the static array
  void* ws = scratch_address();
  if (!ws) return GSPMD_ERR_DEVICE;
  return gspmd_grouped_dot(mesh, dims, lhs_shards, lhs_sh, rhs_shards, rhs_sh, out_shards, out_sh, lhs_fill, epilogue,
                           ws, kScratchBytes, hip_stream);
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_reduce_partials(const void* const* partials, int32_t n_partials, int64_t n_elems,
                              void* out, int32_t out_dtype, void* hip_stream) try {
  if (!partials || !out) return GSPMD_ERR_NULL;
  if (n_partials < 1 || n_partials > kMaxPartials || n_elems < 0) return GSPMD_ERR_BAD_BUFFER;
  if (!is_dtype(out_dtype)) return GSPMD_ERR_UNSUPPORTED;
  for (int i = 0; i < n_partials; ++i) if (!partials[i]) return GSPMD_ERR_NULL;
  return launch_reduce(reinterpret_cast<const float* const*>(partials), n_partials, 1, n_elems, n_elems, out, n_elems,
                       out_dtype, static_cast<hipStream_t>(hip_stream));
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

static int32_t shard_copy(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid, const void* src_global,
                          void* dst_global, const gspmd_shard_buf* shard, uint32_t pad_bits, bool extract, void* hip_stream) try {
  int32_t st = validate_mesh(mesh, nullptr);
  if (st != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, sh)) != GSPMD_OK) return st;
  if ((st = check_buf(shard)) != GSPMD_OK) return st;
  if (has_no_elements(sh)) return GSPMD_OK;   // nothing to copy
  if (!shard->data || (extract ? !src_global : !dst_global)) return GSPMD_ERR_NULL;
  Bounds b;
  if ((st = shard_bounds(mesh, sh, pid, &b)) != GSPMD_OK) return st;
  CopyDesc d;
  std::memset(&d, 0, sizeof(d));
  d.rank = b.rank;
  int64_t total = 1, goff = 0, gs = 1;
  for (int i = b.rank - 1; i >= 0; --i) {
    d.shard[i] = b.shard[i];
    d.valid[i] = b.valid[i];
    d.gstride[i] = gs;
    goff += b.offset[i] * gs;
    gs *= sh->global_shape[i];
    total *= b.shard[i];
  }
  d.sstride[b.rank - 1] = 1;
  if (b.rank >= 2) {
    const int64_t rs = shard->row_stride > 0 ? shard->row_stride : b.shard[b.rank - 1];
    if (rs < b.shard[b.rank - 1]) return GSPMD_ERR_BAD_BUFFER;
    d.sstride[b.rank - 2] = rs;
    for (int i = b.rank - 3; i >= 0; --i) d.sstride[i] = d.sstride[i + 1] * b.shard[i + 1];
  }
  if (total == 0) return GSPMD_OK;
  // A partition wholly in the padding has an offset past the end; it reads/writes nothing
  // of the global tensor, so keep the base pointer in range.
  bool any_valid = true;
  for (int i = 0; i < b.rank; ++i) any_valid = any_valid && b.valid[i] > 0;
  if (!any_valid) goff = 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const unsigned blocks = static_cast<unsigned>(std::min<int64_t>((total + 255) / 256, 256 * 32));
  const dim3 grid(blocks), block(256);
  if (shard->dtype == GSPMD_BF16) {
    typedef bf16_bits T;
    if (extract) hipLaunchKernelGGL((shard_copy_kernel<T, true>), grid, block, 0, stream, d, static_cast<const T*>(src_global) + goff, static_cast<T*>(shard->data), static_cast<T>(pad_bits & 0xffffu), total);
    else hipLaunchKernelGGL((shard_copy_kernel<T, false>), grid, block, 0, stream, d, static_cast<const T*>(shard->data), static_cast<T*>(dst_global) + goff, static_cast<T>(0), total);
  } else {
    typedef uint32_t T;
    if (extract) hipLaunchKernelGGL((shard_copy_kernel<T, true>), grid, block, 0, stream, d, static_cast<const T*>(src_global) + goff, static_cast<T*>(shard->data), pad_bits, total);
    else hipLaunchKernelGGL((shard_copy_kernel<T, false>), grid, block, 0, stream, d, static_cast<const T*>(shard->data), static_cast<T*>(dst_global) + goff, 0u, total);
  }
  return hipGetLastError() == hipSuccess ? GSPMD_OK : GSPMD_ERR_DEVICE;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_shard_extract(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid, const void* global_data,
                            const gspmd_shard_buf* shard, uint32_t pad_bits, void* hip_stream) try {
  return shard_copy(mesh, sh, pid, global_data, nullptr, shard, pad_bits, true, hip_stream);
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_shard_assemble(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid, const gspmd_shard_buf* shard,
                             void* global_data, void* hip_stream) try {
  return shard_copy(mesh, sh, pid, nullptr, global_data, shard, 0, false, hip_stream);
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_reshard_workspace_bytes(const gspmd_mesh* mesh, int64_t* bytes) try {
  if (!bytes) return GSPMD_ERR_NULL;
  int64_t P = 0;
  const int32_t st = validate_mesh(mesh, &P);
  if (st != GSPMD_OK) return st;
  *bytes = round_up(P * 8, kWsAlign) + round_up(P * static_cast<int64_t>(sizeof(ReshardDesc)), kWsAlign);
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_reshard(const gspmd_mesh* mesh, const gspmd_sharding* src_sh, const gspmd_shard_buf* src_shards,
                      const gspmd_sharding* dst_sh, const gspmd_shard_buf* dst_shards,
                      void* workspace, int64_t workspace_bytes, void* hip_stream) try {
  if (!src_shards || !dst_shards) return GSPMD_ERR_NULL;
  int64_t P = 0;
  int32_t st = validate_mesh(mesh, &P);
  if (st != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, src_sh)) != GSPMD_OK || (st = validate_sharding(mesh, dst_sh)) != GSPMD_OK) return st;
  if (src_sh->rank != dst_sh->rank) return GSPMD_ERR_BAD_SHARDING;
  const int rank = src_sh->rank, last = rank - 1;
  for (int i = 0; i < rank; ++i)
    if (src_sh->global_shape[i] != dst_sh->global_shape[i]) return GSPMD_ERR_BAD_SHARDING;
  if (P > 65535) return GSPMD_ERR_UNSUPPORTED;
  // 32-bit index arithmetic in the kernel: a padded dimension (partitions x shard size) must fit
  for (int i = 0; i < rank; ++i)
    if (src_sh->global_shape[i] > (INT32_MAX >> 1)) return GSPMD_ERR_UNSUPPORTED;
  const int32_t dtype = src_shards[0].dtype;
  for (int64_t p = 0; p < P; ++p) {
    if ((st = check_buf(&src_shards[p])) != GSPMD_OK || (st = check_buf(&dst_shards[p])) != GSPMD_OK) return st;
    if (src_shards[p].dtype != dtype || dst_shards[p].dtype != dtype) return GSPMD_ERR_UNSUPPORTED;
    if (src_shards[p].row_stride != src_shards[0].row_stride || dst_shards[p].row_stride != dst_shards[0].row_stride)
      return GSPMD_ERR_BAD_BUFFER;
    if (!has_no_elements(src_sh) && (!src_shards[p].data || !dst_shards[p].data)) return GSPMD_ERR_NULL;
  }
  if (has_no_elements(src_sh)) return GSPMD_OK;   // same global shape on both sides: nothing to move
  int64_t need = 0;
  if ((st = gspmd_reshard_workspace_bytes(mesh, &need)) != GSPMD_OK) return st;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kWsAlign - 1)) || workspace_bytes < need) return GSPMD_ERR_WORKSPACE;

  int64_t mesh_stride[kMaxRank];
  for (int a = mesh->rank - 1, acc = 1; a >= 0; --a) { mesh_stride[a] = acc; acc *= static_cast<int>(mesh->shape[a]); }
  bool src_uses[kMaxRank] = {false};
  for (int i = 0; i < rank; ++i) if (src_sh->dims_mapping[i] >= 0) src_uses[src_sh->dims_mapping[i]] = true;

  // strides of the src shards (one row_stride for all) from any partition's static shape
  Bounds sb0;
  if ((st = shard_bounds(mesh, src_sh, 0, &sb0)) != GSPMD_OK) return st;
  int64_t src_stride[kMaxRank];
  src_stride[last] = 1;
  if (rank >= 2) {
    const int64_t rs = src_shards[0].row_stride > 0 ? src_shards[0].row_stride : sb0.shard[last];
    if (rs < sb0.shard[last]) return GSPMD_ERR_BAD_BUFFER;
    src_stride[rank - 2] = rs;
    for (int i = rank - 3; i >= 0; --i) src_stride[i] = src_stride[i + 1] * sb0.shard[i + 1];
  }

  const size_t esize = dtype == GSPMD_BF16 ? 2 : 4;
  const int vec_elems = static_cast<int>(16 / esize);
  uintptr_t bits = 0;
  for (int64_t p = 0; p < P; ++p) bits |= reinterpret_cast<uintptr_t>(src_shards[p].data) | reinterpret_cast<uintptr_t>(dst_shards[p].data);
  bool vec = !(bits & 15) && sb0.shard[last] % vec_elems == 0;
  for (int i = 0; i < last; ++i) vec = vec && src_stride[i] % vec_elems == 0;

  std::vector<ReshardDesc> descs;
  std::vector<void*> seen;
  int64_t max_rows = 0, max_cols = 0;
  for (int64_t p = 0; p < P; ++p) {
    void* dst = dst_shards[p].data;
    if (std::find(seen.begin(), seen.end(), dst) != seen.end()) continue;   // replicas sharing a buffer: fill it once
    seen.push_back(dst);
    Bounds db;
    if ((st = shard_bounds(mesh, dst_sh, p, &db)) != GSPMD_OK) return st;
    int64_t coords[kMaxRank];
    if ((st = mesh_coords(mesh, p, coords)) != GSPMD_OK) return st;
    ReshardDesc d;
    std::memset(&d, 0, sizeof(d));
    d.dst = dst;
    d.rank = rank;
    int64_t rows = 1, total = 1;
    for (int i = 0; i < rank; ++i) {
      if (db.shard[i] > INT32_MAX) return GSPMD_ERR_UNSUPPORTED;
      d.shard[i] = static_cast<int32_t>(db.shard[i]);
      d.valid[i] = static_cast<int32_t>(db.valid[i]);
      d.dst_off[i] = static_cast<int32_t>(db.offset[i]);
      d.src_per[i] = static_cast<int32_t>(std::max<int64_t>(sb0.shard[i], 1));
      d.src_stride[i] = src_stride[i];
      const int a = src_sh->dims_mapping[i];
      d.pos_stride[i] = a >= 0 ? static_cast<int32_t>(mesh_stride[a]) : 0;
      if (i < last) rows *= db.shard[i];
      total *= db.shard[i];
    }
    for (int a = 0; a < mesh->rank; ++a) if (!src_uses[a]) d.base_pos += static_cast<int32_t>(coords[a] * mesh_stride[a]);
    d.dst_stride[last] = 1;
    if (rank >= 2) {
      const int64_t rs = dst_shards[p].row_stride > 0 ? dst_shards[p].row_stride : db.shard[last];
      if (rs < db.shard[last]) return GSPMD_ERR_BAD_BUFFER;
      d.dst_stride[rank - 2] = rs;
      for (int i = rank - 3; i >= 0; --i) d.dst_stride[i] = d.dst_stride[i + 1] * db.shard[i + 1];
    }
    if (total == 0) continue;
    if (rows > INT32_MAX) return GSPMD_ERR_UNSUPPORTED;
    d.rows = static_cast<int32_t>(rows);
    vec = vec && db.shard[last] % vec_elems == 0;
    for (int i = 0; i < last; ++i) vec = vec && d.dst_stride[i] % vec_elems == 0;
    max_rows = std::max(max_rows, rows);
    max_cols = std::max<int64_t>(max_cols, db.shard[last]);
    descs.push_back(d);
  }
  if (descs.empty()) return GSPMD_OK;

  // tables: [src shard of the partition at each mesh position][descriptors]; as kernel arguments when they fit,
  // else uploaded into the workspace (stream-ordered copy from a temporary host buffer)
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  InlineReshard inl;
  std::memset(&inl, 0, sizeof(inl));
  const void* const* d_ptrs = nullptr;
  const ReshardDesc* d_descs = nullptr;
  if (P <= kInlineReshardSrc && descs.size() <= static_cast<size_t>(kInlineReshardDescs)) {
    for (int64_t pos = 0; pos < P; ++pos) inl.src[pos] = src_shards[mesh->device_ids[pos]].data;
    std::memcpy(inl.d, descs.data(), descs.size() * sizeof(ReshardDesc));
  } else {
    const int64_t ids_bytes = round_up(P * 8, kWsAlign);
    std::vector<char> host(static_cast<size_t>(ids_bytes + descs.size() * sizeof(ReshardDesc)), 0);
    for (int64_t pos = 0; pos < P; ++pos) std::memcpy(host.data() + pos * 8, &src_shards[mesh->device_ids[pos]].data, 8);
    std::memcpy(host.data() + ids_bytes, descs.data(), descs.size() * sizeof(ReshardDesc));
    if (hipMemcpyAsync(workspace, host.data(), host.size(), hipMemcpyHostToDevice, stream) != hipSuccess) return GSPMD_ERR_DEVICE;
    const char* ws = static_cast<const char*>(workspace);
    d_ptrs = reinterpret_cast<const void* const*>(ws);
    d_descs = reinterpret_cast<const ReshardDesc*>(ws + ids_bytes);
  }

  const int v = vec ? vec_elems : 1;
  const int64_t gx = ((max_cols + v - 1) / v + 255) / 256;
  // about 8192 workgroups in all; each thread walks down its column of rows (more, smaller workgroups are slower: 65536 gave 4.2 instead of 5.4 TB/s)
  const int64_t gy = std::min<int64_t>(std::min<int64_t>(max_rows, 65535), std::max<int64_t>(1, 8192 / (gx * static_cast<int64_t>(descs.size()))));
  const dim3 block(256), grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy), static_cast<unsigned>(descs.size()));
  if (dtype == GSPMD_BF16) {
    if (vec) hipLaunchKernelGGL((reshard_kernel<bf16_bits, 8>), grid, block, 0, stream, inl, d_descs, d_ptrs);
    else hipLaunchKernelGGL((reshard_kernel<bf16_bits, 1>), grid, block, 0, stream, inl, d_descs, d_ptrs);
  } else {
    if (vec) hipLaunchKernelGGL((reshard_kernel<uint32_t, 4>), grid, block, 0, stream, inl, d_descs, d_ptrs);
    else hipLaunchKernelGGL((reshard_kernel<uint32_t, 1>), grid, block, 0, stream, inl, d_descs, d_ptrs);
  }
  return hipGetLastError() == hipSuccess ? GSPMD_OK : GSPMD_ERR_DEVICE;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

namespace {

// Roles of the Dot's dimensions without any sharding in play (unit mesh, unsplit tensors).
int32_t dot_roles(const gspmd_dot_dims* dims, const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                  const gspmd_sharding* out_sh, DotRoles* r) {
  const int64_t one = 1, zero = 0;
  gspmd_mesh unit{1, &one, &zero};
  int32_t none[kMaxRank];
  for (int i = 0; i < kMaxRank; ++i) none[i] = -1;
  if (!lhs_sh || !rhs_sh || !out_sh) return GSPMD_ERR_NULL;
  if (lhs_sh->rank > kMaxRank || rhs_sh->rank > kMaxRank || out_sh->rank > kMaxRank) return GSPMD_ERR_BAD_SHARDING;
  gspmd_sharding l{lhs_sh->rank, lhs_sh->global_shape, none}, rr{rhs_sh->rank, rhs_sh->global_shape, none},
      o{out_sh->rank, out_sh->global_shape, none};
  return analyse_dot(&unit, dims, &l, &rr, &o, r, nullptr);
}

int index_in(const int* list, int n, int v) {
  for (int i = 0; i < n; ++i) if (list[i] == v) return i;
  return -1;
}

// Static shard shape and bytes (rows padded to 8 elements) of one partition's temporary under `sh`.
int64_t temp_shard_bytes(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid, size_t esize, int64_t* row_stride) {
  Bounds b;
  if (shard_bounds(mesh, sh, pid, &b) != GSPMD_OK) return -1;
  const int last = b.rank - 1;
  const int64_t ld = round_up(std::max<int64_t>(b.shard[last], 1), 8);
  int64_t rows = 1;
  for (int i = 0; i < last; ++i) rows *= b.shard[i];
  if (row_stride) *row_stride = b.rank >= 2 ? ld : 0;
  return round_up(std::max<int64_t>(rows, 1) * ld * static_cast<int64_t>(esize), kWsAlign);
}

bool same_mapping(const gspmd_sharding* sh, const int32_t* map) {
  for (int i = 0; i < sh->rank; ++i) if (sh->dims_mapping[i] != map[i]) return false;
  return true;
}

// Temporaries of one resharded operand: one buffer per distinct shard position (replicas share), laid out from `base`.
// Returns the bytes used; fills `bufs` (P entries) when base is non-null.
int64_t layout_temps(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t P, int32_t dtype, char* base,
                     std::vector<gspmd_shard_buf>* bufs) {
  const size_t esize = dtype == GSPMD_BF16 ? 2 : 4;
  std::map<std::vector<int64_t>, int64_t> at;     // shard offset -> byte offset of its buffer
  int64_t used = 0;
  for (int64_t p = 0; p < P; ++p) {
    Bounds b;
    if (shard_bounds(mesh, sh, p, &b) != GSPMD_OK) return -1;
    std::vector<int64_t> key(b.offset, b.offset + b.rank);
    int64_t rs = 0;
    const int64_t bytes = temp_shard_bytes(mesh, sh, p, esize, &rs);
    if (bytes < 0) return -1;
    auto it = at.find(key);
    if (it == at.end()) {
      it = at.emplace(key, used).first;
      used += bytes;
    }
    if (bufs) (*bufs)[static_cast<size_t>(p)] = gspmd_shard_buf{base ? base + it->second : nullptr, dtype, rs};
  }
  return used;
}

}  // namespace

int32_t gspmd_compatible_operand_shardings(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                           const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                           const gspmd_sharding* out_sh, int32_t* lhs_mapping, int32_t* rhs_mapping) try {
  if (!lhs_mapping || !rhs_mapping) return GSPMD_ERR_NULL;
  int32_t st = validate_mesh(mesh, nullptr);
  if (st != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, lhs_sh)) != GSPMD_OK || (st = validate_sharding(mesh, rhs_sh)) != GSPMD_OK ||
      (st = validate_sharding(mesh, out_sh)) != GSPMD_OK) return st;
  DotRoles r;
  if ((st = dot_roles(dims, lhs_sh, rhs_sh, out_sh, &r)) != GSPMD_OK) return st;
  for (int i = 0; i < lhs_sh->rank; ++i) lhs_mapping[i] = -1;
  for (int i = 0; i < rhs_sh->rank; ++i) rhs_mapping[i] = -1;
  for (int a = 0; a < mesh->rank; ++a) {
    if (mesh->shape[a] == 1) continue;            // splits nothing
    int ld = -1, rd = -1, od = -1;
    for (int i = 0; i < lhs_sh->rank; ++i) if (lhs_sh->dims_mapping[i] == a) ld = i;
    for (int i = 0; i < rhs_sh->rank; ++i) if (rhs_sh->dims_mapping[i] == a) rd = i;
    for (int i = 0; i < out_sh->rank; ++i) if (out_sh->dims_mapping[i] == a) od = i;
    // a contracting pair split alike on both sides stays: partial sums (scattered if the output is split on it too)
    const int ci = ld >= 0 ? index_in(r.lhs_contract, r.nc, ld) : -1;
    const bool contracting = ci >= 0 && r.rhs_contract[ci] == rd;
    if (contracting) {
      lhs_mapping[ld] = a;
      rhs_mapping[rd] = a;
      continue;
    }
    if (od < 0) continue;                         // output whole on this mesh dimension: so are the operands
    if (od < r.nb) {                              // batch: all three split alike
      lhs_mapping[r.lhs_batch[od]] = a;
      rhs_mapping[r.rhs_batch[od]] = a;
    } else if (od < r.nb + r.nlf) {
      lhs_mapping[r.lhs_free[od - r.nb]] = a;
    } else {
      rhs_mapping[r.rhs_free[od - r.nb - r.nlf]] = a;
    }
  }
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_resharded_dot_workspace_bytes(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                            const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                            const gspmd_sharding* out_sh, int32_t in_dtype, int64_t* bytes) try {
  if (!bytes) return GSPMD_ERR_NULL;
  if (!is_dtype(in_dtype)) return GSPMD_ERR_UNSUPPORTED;
  int32_t lmap[kMaxRank], rmap[kMaxRank];
  int32_t st = gspmd_compatible_operand_shardings(mesh, dims, lhs_sh, rhs_sh, out_sh, lmap, rmap);
  if (st != GSPMD_OK) return st;
  int64_t P = 0;
  if ((st = validate_mesh(mesh, &P)) != GSPMD_OK) return st;
  const gspmd_sharding l2{lhs_sh->rank, lhs_sh->global_shape, lmap}, r2{rhs_sh->rank, rhs_sh->global_shape, rmap};
  int64_t total = 0, n = 0;
  if ((st = gspmd_reshard_workspace_bytes(mesh, &n)) != GSPMD_OK) return st;
  total += 2 * n;
  if (!same_mapping(lhs_sh, lmap)) {
    if ((n = layout_temps(mesh, &l2, P, in_dtype, nullptr, nullptr)) < 0) return GSPMD_ERR_UNSUPPORTED;
    total += n;
  }
  if (!same_mapping(rhs_sh, rmap)) {
    if ((n = layout_temps(mesh, &r2, P, in_dtype, nullptr, nullptr)) < 0) return GSPMD_ERR_UNSUPPORTED;
    total += n;
  }
  if ((st = gspmd_dot_workspace_bytes(mesh, dims, &l2, &r2, out_sh, -1, 1, &n)) != GSPMD_OK) return st;
  *bytes = total + n;
  return GSPMD_OK;
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_resharded_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                            const gspmd_shard_buf* lhs_shards, const gspmd_sharding* lhs_sh,
                            const gspmd_shard_buf* rhs_shards, const gspmd_sharding* rhs_sh,
                            const gspmd_shard_buf* out_shards, const gspmd_sharding* out_sh,
                            const int64_t* lhs_fill, int32_t epilogue,
                            void* workspace, int64_t workspace_bytes, void* hip_stream) try {
  if (!lhs_shards || !rhs_shards || !out_shards) return GSPMD_ERR_NULL;
  int32_t lmap[kMaxRank], rmap[kMaxRank];
  int32_t st = gspmd_compatible_operand_shardings(mesh, dims, lhs_sh, rhs_sh, out_sh, lmap, rmap);
  if (st != GSPMD_OK) return st;
  int64_t P = 0;
  if ((st = validate_mesh(mesh, &P)) != GSPMD_OK) return st;
  if ((st = check_buf(&lhs_shards[0])) != GSPMD_OK || (st = check_buf(&rhs_shards[0])) != GSPMD_OK) return st;
  const int32_t in_dtype = lhs_shards[0].dtype;
  if (rhs_shards[0].dtype != in_dtype) return GSPMD_ERR_UNSUPPORTED;
  int64_t need = 0;
  if ((st = gspmd_resharded_dot_workspace_bytes(mesh, dims, lhs_sh, rhs_sh, out_sh, in_dtype, &need)) != GSPMD_OK) return st;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kWsAlign - 1)) || workspace_bytes < need) return GSPMD_ERR_WORKSPACE;
  const gspmd_sharding l2{lhs_sh->rank, lhs_sh->global_shape, lmap}, r2{rhs_sh->rank, rhs_sh->global_shape, rmap};
  char* ws = static_cast<char*>(workspace);
  int64_t rs_bytes = 0;
  if ((st = gspmd_reshard_workspace_bytes(mesh, &rs_bytes)) != GSPMD_OK) return st;
  char* rs_ws[2] = {ws, ws + rs_bytes};
  ws += 2 * rs_bytes;
  std::vector<gspmd_shard_buf> ltmp(static_cast<size_t>(P)), rtmp(static_cast<size_t>(P));
  const gspmd_shard_buf* luse = lhs_shards;
  const gspmd_shard_buf* ruse = rhs_shards;
  if (!same_mapping(lhs_sh, lmap)) {
    const int64_t n = layout_temps(mesh, &l2, P, in_dtype, ws, &ltmp);
    if (n < 0) return GSPMD_ERR_UNSUPPORTED;
    ws += n;
    if ((st = gspmd_reshard(mesh, lhs_sh, lhs_shards, &l2, ltmp.data(), rs_ws[0], rs_bytes, hip_stream)) != GSPMD_OK) return st;
    luse = ltmp.data();
  }
  if (!same_mapping(rhs_sh, rmap)) {
    const int64_t n = layout_temps(mesh, &r2, P, in_dtype, ws, &rtmp);
    if (n < 0) return GSPMD_ERR_UNSUPPORTED;
    ws += n;
    if ((st = gspmd_reshard(mesh, rhs_sh, rhs_shards, &r2, rtmp.data(), rs_ws[1], rs_bytes, hip_stream)) != GSPMD_OK) return st;
    ruse = rtmp.data();
  }
  const int64_t left = workspace_bytes - (ws - static_cast<char*>(workspace));
  return gspmd_grouped_dot(mesh, dims, luse, &l2, ruse, &r2, out_shards, out_sh, lhs_fill, epilogue, ws, left, hip_stream);
} catch (...) { return GSPMD_ERR_HOST_MEMORY; }

int32_t gspmd_set_tile_timeline(void* device_records, int64_t n_records) try {
  if (n_records < 0 || n_records > INT32_MAX) return GSPMD_ERR_BAD_BUFFER;
  if (device_records == nullptr || n_records == 0) {
    g_timeline.store(nullptr, std::memory_order_release);
    g_timeline_records.store(0, std::memory_order_release);
    return GSPMD_OK;
  }
  if (reinterpret_cast<uintptr_t>(device_records) & 7) return GSPMD_ERR_BAD_BUFFER;
  g_timeline_records.store(static_cast<int>(n_records), std::memory_order_release);
  g_timeline.store(static_cast<unsigned long long*>(device_records), std::memory_order_release);
  return GSPMD_OK;
} catch (...) {
  return GSPMD_ERR_HOST_MEMORY;
}

}  // extern "C"
