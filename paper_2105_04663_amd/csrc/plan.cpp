// Host index math: see plan.h.
#include "plan.h"

#include <algorithm>
#include <cstring>

namespace gspmd {

int32_t validate_mesh(const gspmd_mesh* mesh, int64_t* n_partitions) {
  if (!mesh || !mesh->shape || !mesh->device_ids) return GSPMD_ERR_NULL;
  if (mesh->rank <= 0 || mesh->rank > kMaxRank) return GSPMD_ERR_BAD_MESH;
  int64_t p = 1;
  for (int i = 0; i < mesh->rank; ++i) {
    if (mesh->shape[i] <= 0) return GSPMD_ERR_BAD_MESH;
    if (p > kMaxPartitions / mesh->shape[i]) return GSPMD_ERR_BAD_MESH;   // bounds the host tables built per partition
    p *= mesh->shape[i];
  }
  // ids must be a permutation of 0..P-1 (every partition owns exactly one mesh position)
  std::vector<uint8_t> seen(static_cast<size_t>(p), 0);
  for (int64_t i = 0; i < p; ++i) {
    int64_t d = mesh->device_ids[i];
    if (d < 0 || d >= p || seen[static_cast<size_t>(d)]) return GSPMD_ERR_BAD_MESH;
    seen[static_cast<size_t>(d)] = 1;
  }
  if (n_partitions) *n_partitions = p;
  return GSPMD_OK;
}

int32_t validate_sharding(const gspmd_mesh* mesh, const gspmd_sharding* sh) {
  if (!sh || !sh->global_shape || !sh->dims_mapping) return GSPMD_ERR_NULL;
  if (sh->rank <= 0 || sh->rank > kMaxRank) return GSPMD_ERR_BAD_SHARDING;
  bool used[kMaxRank] = {false};
  for (int i = 0; i < sh->rank; ++i) {
    if (sh->global_shape[i] < 0) return GSPMD_ERR_BAD_SHARDING;
    int a = sh->dims_mapping[i];
    if (a == -1) continue;
    if (a < 0 || a >= mesh->rank) return GSPMD_ERR_BAD_SHARDING;
    if (used[a]) return GSPMD_ERR_BAD_SHARDING;  // a mesh dimension appears at most once
    used[a] = true;
  }
  return GSPMD_OK;
}

int32_t mesh_coords(const gspmd_mesh* mesh, int64_t pid, int64_t* coords) {
  int64_t p = 1;
  for (int i = 0; i < mesh->rank; ++i) p *= mesh->shape[i];
  if (pid < 0 || pid >= p) return GSPMD_ERR_PARTITION_RANGE;
  int64_t lin = -1;
  for (int64_t i = 0; i < p; ++i)
    if (mesh->device_ids[i] == pid) { lin = i; break; }
  if (lin < 0) return GSPMD_ERR_PARTITION_RANGE;
  for (int i = mesh->rank - 1; i >= 0; --i) {
    coords[i] = lin % mesh->shape[i];
    lin /= mesh->shape[i];
  }
  return GSPMD_OK;
}

int32_t shard_bounds(const gspmd_mesh* mesh, const gspmd_sharding* sh, int64_t pid, Bounds* b) {
  int64_t coords[kMaxRank];
  int32_t st = mesh_coords(mesh, pid, coords);
  if (st != GSPMD_OK) return st;
  b->rank = sh->rank;
  for (int i = 0; i < sh->rank; ++i) {
    const int64_t D = sh->global_shape[i];
    const int a = sh->dims_mapping[i];
    if (a == -1) {
      b->offset[i] = 0; b->valid[i] = D; b->shard[i] = D;
      continue;
    }
    const int64_t n = mesh->shape[a];
    const int64_t per = (D + n - 1) / n;          // static shard size, same for every partition
    const int64_t off = coords[a] * per;          // not clamped: pure function of the partition id
    b->shard[i] = per;
    b->offset[i] = off;
    b->valid[i] = std::max<int64_t>(0, std::min<int64_t>(per, D - off));
  }
  return GSPMD_OK;
}

namespace {

int find_axis_dim(const gspmd_sharding* sh, int axis) {
  for (int i = 0; i < sh->rank; ++i) if (sh->dims_mapping[i] == axis) return i;
  return -1;
}

int index_of(const int* list, int n, int v) {
  for (int i = 0; i < n; ++i) if (list[i] == v) return i;
  return -1;
}

}  // namespace

int32_t analyse_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                    const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                    const gspmd_sharding* out_sh, DotRoles* r, int32_t* axis_class) {
  if (!dims) return GSPMD_ERR_NULL;
  int32_t st = validate_mesh(mesh, nullptr);
  if (st != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, lhs_sh)) != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, rhs_sh)) != GSPMD_OK) return st;
  if ((st = validate_sharding(mesh, out_sh)) != GSPMD_OK) return st;
  const int nb = dims->n_batch, nc = dims->n_contract;
  if (nb < 0 || nc < 0 || nb + nc > kMaxRank) return GSPMD_ERR_BAD_DOT_DIMS;
  if (nb > 0 && (!dims->lhs_batch || !dims->rhs_batch)) return GSPMD_ERR_NULL;
  if (nc > 0 && (!dims->lhs_contract || !dims->rhs_contract)) return GSPMD_ERR_NULL;
  const int lr = lhs_sh->rank, rr = rhs_sh->rank;
  if (nb + nc > lr || nb + nc > rr) return GSPMD_ERR_BAD_DOT_DIMS;
  r->nb = nb; r->nc = nc;
  bool lused[kMaxRank] = {false}, rused[kMaxRank] = {false};
  for (int i = 0; i < nb; ++i) {
    int a = dims->lhs_batch[i], b = dims->rhs_batch[i];
    if (a < 0 || a >= lr || b < 0 || b >= rr || lused[a] || rused[b]) return GSPMD_ERR_BAD_DOT_DIMS;
    if (lhs_sh->global_shape[a] != rhs_sh->global_shape[b]) return GSPMD_ERR_BAD_DOT_DIMS;
    lused[a] = rused[b] = true;
    r->lhs_batch[i] = a; r->rhs_batch[i] = b;
  }
  std::vector<std::pair<int, int>> cp;
  for (int i = 0; i < nc; ++i) {
    int a = dims->lhs_contract[i], b = dims->rhs_contract[i];
    if (a < 0 || a >= lr || b < 0 || b >= rr || lused[a] || rused[b]) return GSPMD_ERR_BAD_DOT_DIMS;
    if (lhs_sh->global_shape[a] != rhs_sh->global_shape[b]) return GSPMD_ERR_BAD_DOT_DIMS;
    lused[a] = rused[b] = true;
    cp.emplace_back(a, b);
  }
  std::sort(cp.begin(), cp.end());   // a sum does not depend on the order of its dimensions
  for (int i = 0; i < nc; ++i) { r->lhs_contract[i] = cp[i].first; r->rhs_contract[i] = cp[i].second; }
  r->nlf = r->nrf = 0;
  for (int i = 0; i < lr; ++i) if (!lused[i]) r->lhs_free[r->nlf++] = i;
  for (int i = 0; i < rr; ++i) if (!rused[i]) r->rhs_free[r->nrf++] = i;
  // output shape: batch, lhs free, rhs free
  if (out_sh->rank != nb + r->nlf + r->nrf) return GSPMD_ERR_BAD_DOT_DIMS;
  for (int i = 0; i < nb; ++i)
    if (out_sh->global_shape[i] != lhs_sh->global_shape[r->lhs_batch[i]]) return GSPMD_ERR_BAD_DOT_DIMS;
  for (int i = 0; i < r->nlf; ++i)
    if (out_sh->global_shape[nb + i] != lhs_sh->global_shape[r->lhs_free[i]]) return GSPMD_ERR_BAD_DOT_DIMS;
  for (int i = 0; i < r->nrf; ++i)
    if (out_sh->global_shape[nb + r->nlf + i] != rhs_sh->global_shape[r->rhs_free[i]]) return GSPMD_ERR_BAD_DOT_DIMS;

  // Per mesh dimension: which of the communication-free patterns it carries.
  for (int a = 0; a < mesh->rank; ++a) {
    const int ld = find_axis_dim(lhs_sh, a), rd = find_axis_dim(rhs_sh, a), od = find_axis_dim(out_sh, a);
    int cls = -1;
    // A mesh dimension of size 1 splits nothing: whatever is mapped to it is whole (in particular a contracting
    // dimension mapped to it needs no partial sums).
    if (mesh->shape[a] == 1 || (ld < 0 && rd < 0 && od < 0)) {
      cls = GSPMD_AXIS_UNUSED;
    } else if (ld >= 0 && rd >= 0 && od >= 0) {
      const int bi = index_of(r->lhs_batch, nb, ld);
      const int ci = index_of(r->lhs_contract, nc, ld);
      if (bi >= 0 && r->rhs_batch[bi] == rd && od == bi) cls = GSPMD_AXIS_BATCH;
      // a contracting pair and, independently, some out dimension: the sum is scattered along that dimension
      else if (ci >= 0 && r->rhs_contract[ci] == rd) cls = GSPMD_AXIS_CONTRACTING_SCATTER;
    } else if (ld >= 0 && rd < 0 && od >= 0) {
      const int fi = index_of(r->lhs_free, r->nlf, ld);
      if (fi >= 0 && od == nb + fi) cls = GSPMD_AXIS_LHS_FREE;
    } else if (ld < 0 && rd >= 0 && od >= 0) {
      const int fi = index_of(r->rhs_free, r->nrf, rd);
      if (fi >= 0 && od == nb + r->nlf + fi) cls = GSPMD_AXIS_RHS_FREE;
    } else if (ld >= 0 && rd >= 0 && od < 0) {
      const int ci = index_of(r->lhs_contract, nc, ld);
      if (ci >= 0 && r->rhs_contract[ci] == rd) cls = GSPMD_AXIS_CONTRACTING;
    }
    if (cls < 0) return GSPMD_ERR_NEEDS_RESHARD;
    if (axis_class) axis_class[a] = cls;
  }
  return GSPMD_OK;
}

namespace {

// Strides (in elements) of a shard buffer with static shape `shard`.
int32_t shard_strides(const Bounds& b, int64_t row_stride, int64_t* stride) {
  const int r = b.rank;
  stride[r - 1] = 1;
  if (r >= 2) {
    int64_t rs = row_stride > 0 ? row_stride : b.shard[r - 1];
    if (rs < b.shard[r - 1]) return GSPMD_ERR_BAD_BUFFER;
    stride[r - 2] = rs;
    for (int i = r - 3; i >= 0; --i) stride[i] = stride[i + 1] * b.shard[i + 1];
  }
  return GSPMD_OK;
}

struct Layout {
  // flattened inner extent + the outer dims enumerated one by one
  int64_t inner_static = 1, inner_valid = 1;
  int n_outer = 0;
  int outer_dim_op[kMaxRank], outer_dim_out[kMaxRank];
};

// Flatten the dims of one free group (outer -> inner) as far as both tensors allow:
// a suffix flattens if every dim inside it but the outermost is fully valid and the
// strides nest densely in the operand and in the output.
Layout flatten_free(const int* op_dims, int n, int out_first, const Bounds& ob, const int64_t* ostride,
                    const Bounds& cb, const int64_t* cstride) {
  Layout l;
  if (n == 0) return l;
  int j = n - 1;
  l.inner_static = ob.shard[op_dims[j]];
  l.inner_valid = ob.valid[op_dims[j]];
  while (j > 0) {
    const int d = op_dims[j], dprev = op_dims[j - 1];
    const int c = out_first + j, cprev = out_first + j - 1;
    const bool full = ob.valid[d] == ob.shard[d];
    const bool nest_op = ostride[dprev] == ostride[d] * ob.shard[d];
    const bool nest_out = cstride[cprev] == cstride[c] * cb.shard[c];
    if (!(full && nest_op && nest_out)) break;
    --j;
    l.inner_valid = ob.valid[op_dims[j]] * l.inner_static;
    l.inner_static *= ob.shard[op_dims[j]];
  }
  for (int i = 0; i < j; ++i) {
    l.outer_dim_op[l.n_outer] = op_dims[i];
    l.outer_dim_out[l.n_outer] = out_first + i;
    ++l.n_outer;
  }
  return l;
}

size_t dtype_size(int32_t dt) { return dt == GSPMD_BF16 ? 2 : 4; }

}  // namespace

int32_t plan_partition(const gspmd_mesh* mesh, const DotRoles& r,
                       const gspmd_shard_buf* lhs, const gspmd_sharding* lhs_sh,
                       const gspmd_shard_buf* rhs, const gspmd_sharding* rhs_sh,
                       const gspmd_shard_buf* out, const gspmd_sharding* out_sh,
                       int64_t pid, const int64_t* lhs_fill, void* c_override,
                       std::vector<Problem>* problems, int64_t* out_static_elems, int32_t* layout) {
  Bounds lb, rb, ob;
  int32_t st;
  if ((st = shard_bounds(mesh, lhs_sh, pid, &lb)) != GSPMD_OK) return st;
  if ((st = shard_bounds(mesh, rhs_sh, pid, &rb)) != GSPMD_OK) return st;
  if ((st = shard_bounds(mesh, out_sh, pid, &ob)) != GSPMD_OK) return st;
  const int nb = r.nb, nc = r.nc, lr = lhs_sh->rank, rr = rhs_sh->rank;

  // Supported dimension orders: the last (contiguous) dimension of each operand is its innermost
  // contracting dimension (K contiguous) or its innermost non-contracting dimension (K-major),
  // and the contracting dimensions nest alike in both operands (checked on the strides below).
  // The forward einsums are lhs K-contiguous x rhs K-major; a weight gradient (tokens contract)
  // is K-major x K-major, an input gradient K-contiguous x K-contiguous.
  if (nc == 0) return GSPMD_ERR_UNSUPPORTED;
  const bool a_kc = r.lhs_contract[nc - 1] == lr - 1;
  const bool a_km = r.nlf > 0 && r.lhs_free[r.nlf - 1] == lr - 1;
  const bool b_kc = r.rhs_contract[nc - 1] == rr - 1;
  const bool b_km = r.nrf > 0 && r.rhs_free[r.nrf - 1] == rr - 1;
  if (!(a_kc || a_km) || !(b_kc || b_km)) return GSPMD_ERR_UNSUPPORTED;   // a batch dimension is the contiguous one
  if (layout) *layout = (a_km ? GSPMD_LAYOUT_LHS_K_MAJOR : 0) | (b_kc ? GSPMD_LAYOUT_RHS_K_CONTIGUOUS : 0);

  int64_t ls[kMaxRank], rs[kMaxRank], cs[kMaxRank];
  if ((st = shard_strides(lb, lhs->row_stride, ls)) != GSPMD_OK) return st;
  if ((st = shard_strides(rb, rhs->row_stride, rs)) != GSPMD_OK) return st;
  int64_t c_row_stride = c_override ? 0 : out->row_stride;
  if ((st = shard_strides(ob, c_row_stride, cs)) != GSPMD_OK) return st;

  int64_t out_elems = 1;
  for (int i = 0; i < ob.rank; ++i) out_elems *= ob.shard[i];
  if (out_static_elems) *out_static_elems = out_elems;

  // Contracting dims flatten to one K: inner ones must be whole and dense in the lhs.
  int64_t Ks = 1, Kv = 1;
  for (int i = nc - 1; i >= 0; --i) {
    const int ld = r.lhs_contract[i], rd = r.rhs_contract[i];
    if (lb.valid[ld] != rb.valid[rd] || lb.shard[ld] != rb.shard[rd]) return GSPMD_ERR_NEEDS_RESHARD;
    if (i < nc - 1) {
      const int ldn = r.lhs_contract[i + 1], rdn = r.rhs_contract[i + 1];
      if (lb.valid[ldn] != lb.shard[ldn]) return GSPMD_ERR_UNSUPPORTED;
      if (ls[ld] != ls[ldn] * lb.shard[ldn]) return GSPMD_ERR_UNSUPPORTED;
      if (rs[rd] != rs[rdn] * rb.shard[rdn]) return GSPMD_ERR_UNSUPPORTED;
    }
    Kv = (i == nc - 1) ? lb.valid[ld] : lb.valid[ld] * Ks;
    Ks *= lb.shard[ld];
  }
  const Layout lm = flatten_free(r.lhs_free, r.nlf, nb, lb, ls, ob, cs);
  const Layout ln = flatten_free(r.rhs_free, r.nrf, nb + r.nlf, rb, rs, ob, cs);

  // leading dimensions of the flattened views: the stride of whichever index is not contiguous
  const int64_t lda = a_km ? ls[r.lhs_contract[nc - 1]] : (r.nlf ? ls[r.lhs_free[r.nlf - 1]] : Ks);
  const int64_t ldb = b_km ? rs[r.rhs_contract[nc - 1]] : (r.nrf ? rs[r.rhs_free[r.nrf - 1]] : Ks);
  const int64_t ldc = r.nlf ? cs[nb + r.nlf - 1] : ln.inner_static;
  const int64_t lim = INT32_MAX;
  if (lm.inner_static > lim || ln.inner_static > lim || Ks > lim || lda > lim || ldb > lim || ldc > lim)
    return GSPMD_ERR_UNSUPPORTED;
  // Fill counts apply to the first lhs dimension that is not a batch dimension (the capacity dimension of the
  // mixture-of-experts einsums).  Non-contracting: it must be the only one (its rows are clamped).  Contracting (the
  // experts' weight gradient): it must be the outermost contracting dimension (the valid K is clamped).
  int fill_dim = -1;
  bool fill_contracts = false;
  if (lhs_fill) {
    for (int i = 0; i < lr && fill_dim < 0; ++i) {
      bool is_batch = false;
      for (int j = 0; j < nb; ++j) is_batch = is_batch || r.lhs_batch[j] == i;
      if (!is_batch) fill_dim = i;
    }
    if (fill_dim < 0) return GSPMD_ERR_UNSUPPORTED;
    fill_contracts = r.lhs_contract[0] == fill_dim;
    if (!fill_contracts && !(r.nlf == 1 && r.lhs_free[0] == fill_dim)) return GSPMD_ERR_UNSUPPORTED;
  }
  const int64_t k_inner = lb.shard[r.lhs_contract[0]] ? Ks / lb.shard[r.lhs_contract[0]] : 0;   // K positions per index of the outermost contracting dim

  // enumerate: batch entries x outer lhs-free x outer rhs-free (static extents, so that every
  // output element of the static shard is written)
  int n_loop = 0;
  int64_t extent[3 * kMaxRank], valid[3 * kMaxRank], sa[3 * kMaxRank], sb[3 * kMaxRank], sc[3 * kMaxRank];
  int64_t goff[3 * kMaxRank], gsize[3 * kMaxRank];   // global offset/size of batch dims (for fill lookup)
  for (int i = 0; i < nb; ++i) {
    const int ld = r.lhs_batch[i], rd = r.rhs_batch[i];
    extent[n_loop] = lb.shard[ld]; valid[n_loop] = lb.valid[ld];
    if (lb.valid[ld] != rb.valid[rd] || lb.valid[ld] != ob.valid[i]) return GSPMD_ERR_NEEDS_RESHARD;
    sa[n_loop] = ls[ld]; sb[n_loop] = rs[rd]; sc[n_loop] = cs[i];
    goff[n_loop] = lb.offset[ld]; gsize[n_loop] = lhs_sh->global_shape[ld];
    ++n_loop;
  }
  for (int i = 0; i < lm.n_outer; ++i) {
    const int d = lm.outer_dim_op[i];
    extent[n_loop] = lb.shard[d]; valid[n_loop] = lb.valid[d];
    sa[n_loop] = ls[d]; sb[n_loop] = 0; sc[n_loop] = cs[lm.outer_dim_out[i]];
    ++n_loop;
  }
  for (int i = 0; i < ln.n_outer; ++i) {
    const int d = ln.outer_dim_op[i];
    extent[n_loop] = rb.shard[d]; valid[n_loop] = rb.valid[d];
    sa[n_loop] = 0; sb[n_loop] = rs[d]; sc[n_loop] = cs[ln.outer_dim_out[i]];
    ++n_loop;
  }
  int64_t total = 1;
  for (int i = 0; i < n_loop; ++i) {
    if (extent[i] == 0) { total = 0; break; }
    if (total > kMaxProblems / extent[i]) return GSPMD_ERR_UNSUPPORTED;
    total *= extent[i];
  }
  if (lm.inner_static == 0 || ln.inner_static == 0) total = 0;   // nothing to write
  if (static_cast<int64_t>(problems->size()) + total > kMaxProblems) return GSPMD_ERR_UNSUPPORTED;

  const size_t ea = dtype_size(lhs->dtype), eb = dtype_size(rhs->dtype);
  const size_t ec = c_override ? 4 : dtype_size(out->dtype);
  char* cbase = static_cast<char*>(c_override ? c_override : out->data);
  int64_t idx[3 * kMaxRank] = {0};
  for (int64_t t = 0; t < total; ++t) {
    int64_t oa = 0, obb = 0, oc = 0;
    bool live = true;
    for (int i = 0; i < n_loop; ++i) {
      oa += idx[i] * sa[i]; obb += idx[i] * sb[i]; oc += idx[i] * sc[i];
      if (idx[i] >= valid[i]) live = false;
    }
    Problem p;
    std::memset(&p, 0, sizeof(p));
    p.A = static_cast<const char*>(lhs->data) + oa * static_cast<int64_t>(ea);
    p.B = static_cast<const char*>(rhs->data) + obb * static_cast<int64_t>(eb);
    p.C = cbase + oc * static_cast<int64_t>(ec);
    int64_t mv = live ? lm.inner_valid : 0, kv = live ? Kv : 0;
    if (live && lhs_fill) {
      int64_t g = 0;   // row-major index over the GLOBAL batch dims
      for (int i = 0; i < nb; ++i) g = g * gsize[i] + (goff[i] + idx[i]);
      const int64_t f = lhs_fill[g];
      if (f < 0) return GSPMD_ERR_BAD_BUFFER;
      const int64_t occupied = std::max<int64_t>(0, f - lb.offset[fill_dim]);   // of this shard's positions
      if (fill_contracts) kv = std::min<int64_t>(kv, occupied * k_inner);
      else mv = std::min<int64_t>(mv, occupied);
    }
    p.Mv = static_cast<int32_t>(mv);
    p.Nv = static_cast<int32_t>(live ? ln.inner_valid : 0);
    p.Kv = static_cast<int32_t>(kv);
    p.Ms = static_cast<int32_t>(lm.inner_static);
    p.Ns = static_cast<int32_t>(ln.inner_static);
    p.lda = static_cast<int32_t>(lda); p.ldb = static_cast<int32_t>(ldb); p.ldc = static_cast<int32_t>(ldc);
    if (p.Mv == 0 || p.Nv == 0 || p.Kv == 0) { p.Mv = p.Nv = p.Kv = 0; }
    problems->push_back(p);
    for (int i = n_loop - 1; i >= 0; --i) {   // odometer
      if (++idx[i] < extent[i]) break;
      idx[i] = 0;
    }
  }
  return GSPMD_OK;
}

int32_t count_partition(const gspmd_mesh* mesh, const DotRoles& r,
                        const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                        const gspmd_sharding* out_sh, int64_t pid,
                        int64_t* n_problems, int64_t* out_static_elems, int64_t* max_tiles, int tile) {
  // Upper bound that does not depend on the buffers: every batch entry and every index of
  // the free dims except the innermost one of each side may become a problem of its own.
  Bounds lb, rb, ob;
  int32_t st;
  if ((st = shard_bounds(mesh, lhs_sh, pid, &lb)) != GSPMD_OK) return st;
  if ((st = shard_bounds(mesh, rhs_sh, pid, &rb)) != GSPMD_OK) return st;
  if ((st = shard_bounds(mesh, out_sh, pid, &ob)) != GSPMD_OK) return st;
  int64_t n = 1;
  auto mul = [&](int64_t e) -> bool {
    if (e <= 0) { n = 0; return true; }
    if (n > kMaxProblems / e) return false;
    n *= e; return true;
  };
  for (int i = 0; i < r.nb; ++i) if (!mul(lb.shard[r.lhs_batch[i]])) return GSPMD_ERR_UNSUPPORTED;
  for (int i = 0; i + 1 < r.nlf; ++i) if (!mul(lb.shard[r.lhs_free[i]])) return GSPMD_ERR_UNSUPPORTED;
  for (int i = 0; i + 1 < r.nrf; ++i) if (!mul(rb.shard[r.rhs_free[i]])) return GSPMD_ERR_UNSUPPORTED;
  int64_t e = 1;
  for (int i = 0; i < ob.rank; ++i) e *= ob.shard[i];
  *n_problems = n;
  *out_static_elems = e;
  if (max_tiles) {
    const int64_t im = r.nlf ? lb.shard[r.lhs_free[r.nlf - 1]] : 1, in = r.nrf ? rb.shard[r.rhs_free[r.nrf - 1]] : 1;
    const int64_t tm = (im + tile - 1) / tile, tn = (in + tile - 1) / tile, cap = int64_t(1) << 40;
    *max_tiles = (tm > cap / std::max<int64_t>(tn, 1) || n > cap / std::max<int64_t>(tm * tn, 1)) ? cap : n * tm * tn;
  }
  return GSPMD_OK;
}

}  // namespace gspmd
