/*
 * gspmd.h -- C ABI of the MI355X (gfx950) per-partition einsum library.
 *
 * The library executes the piece of a GSPMD-partitioned program that every
 * partition runs locally for a Dot/Einsum: the contraction on that partition's
 * shards (Section 3.2, Section 4), with uneven dimensions padded to a static
 * shard size and masked (Section 4.1).  Mesh partitions are *virtual*: all of
 * them live on one GPU; there is no communication.  The one exchange the method
 * needs -- the AllReduce along a mesh dimension that splits a contracting
 * dimension (Section 4.2) -- is stood in for by an on-GPU sum of partials.
 *
 * Conventions for every entry point
 *   - Plain C types only.  "host" pointers are read during the call and not
 *     kept.  "device" pointers are HIP device memory owned by the caller; the
 *     library never allocates or frees device memory.
 *   - Device work is enqueued on the given hipStream_t (passed as void*; NULL
 *     is the default stream) and is complete when that stream is.
 *   - Every function returns a gspmd_status and never throws (a failed host allocation comes back as
 *     GSPMD_ERR_HOST_MEMORY), aborts or prints.  Outputs are written only on GSPMD_OK.
 *   - The library keeps no state between calls (gspmd_grouped_dot_noalloc's static workspace and the profiling switch
 *     of gspmd_set_tile_timeline aside); independent calls may be made from several host threads.
 *   - HIP graphs: a kernel-launching call whose launch tables fit its kernels' arguments enqueues kernels only and
 *     may be recorded into a graph: a Dot lowered to at most 32 GEMM problems (every benchmark configuration; the
 *     count is what gspmd_plan_dot reports, summed over the partitions of a grouped call), a resharding on a mesh of
 *     at most 64 partitions with at most 8 distinct destination buffers.  Beyond that the tables are uploaded into
 *     the workspace with a stream-ordered copy from a temporary host buffer, and such a call must not be recorded.
 *   - Tensors are row-major.  A shard buffer has the STATIC shard shape (ceil(D/n) per split dimension,
 *     Section 4.1), whatever the partition's valid length.  Padding may hold anything, including NaN: no value at
 *     an index >= the valid length of any dimension reaches a result.  Reads stay inside the rows of the valid
 *     region: the MFMA kernels load 16 bytes at a time, so when a row's valid length is not a multiple of 8 elements
 *     the chunk that holds its last valid elements is loaded whole (from inside the row's own allocation, which the
 *     required row stride of a multiple of 8 elements guarantees) and the excess is discarded or zeroed in
 *     registers.  The padded part of outputs is written as zeros.
 */
#ifndef GSPMD_H_
#define GSPMD_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GSPMD_OK = 0,
  GSPMD_ERR_NULL = 1,            /* a required pointer is NULL */
  GSPMD_ERR_BAD_MESH = 2,        /* rank/size <= 0, more than 2^20 partitions, ids not a permutation of 0..P-1 */
  GSPMD_ERR_BAD_SHARDING = 3,    /* rank mismatch, mesh dim out of range or used twice (Section 3.1) */
  GSPMD_ERR_PARTITION_RANGE = 4, /* partition id not in the mesh */
  GSPMD_ERR_BAD_DOT_DIMS = 5,    /* duplicate/out-of-range dims, size mismatch, wrong output shape */
  GSPMD_ERR_NEEDS_RESHARD = 6,   /* shardings are not one of the communication-free cases (Section 4.5) */
  GSPMD_ERR_UNSUPPORTED = 7,     /* dtype/layout combination not implemented */
  GSPMD_ERR_WORKSPACE = 8,       /* workspace missing, misaligned or too small */
  GSPMD_ERR_DEVICE = 9,          /* a HIP call failed */
  GSPMD_ERR_BAD_BUFFER = 10,     /* row_stride smaller than the shard's last dimension, bad fill count */
  GSPMD_ERR_HOST_MEMORY = 11     /* a host-side allocation failed */
} gspmd_status;

typedef enum { GSPMD_F32 = 0, GSPMD_BF16 = 1 } gspmd_dtype;

/* How a mesh dimension is used by one Dot (Section 3.2 taxonomy applied per mesh dimension,
 * the cases matched recursively in Section 4.4). */
typedef enum {
  GSPMD_AXIS_UNUSED = 0,      /* no operand or output dimension is split on it (replicated); always the class of a
                                 mesh dimension of size 1, which splits nothing whatever is mapped to it */
  GSPMD_AXIS_BATCH = 1,       /* the same batch dimension of lhs, rhs and out */
  GSPMD_AXIS_LHS_FREE = 2,    /* a non-contracting lhs dimension and the matching out dimension */
  GSPMD_AXIS_RHS_FREE = 3,    /* a non-contracting rhs dimension and the matching out dimension */
  GSPMD_AXIS_CONTRACTING = 4, /* the same contracting dimension of lhs and rhs; out holds a partial sum */
  GSPMD_AXIS_CONTRACTING_SCATTER = 5 /* as CONTRACTING, and an out dimension is split on it too: after the sum every
                                        partition keeps its slice (ReduceScatter = AllReduce + DynamicSlice, Section 4.2) */
} gspmd_axis_class;

/* Elementwise function applied to the finished sum before it is stored (the feed-forward layer of Section 5.1 is
 * Relu(x W_in) W_out). */
typedef enum { GSPMD_EPILOGUE_NONE = 0, GSPMD_EPILOGUE_RELU = 1 } gspmd_epilogue;

/* Device mesh (Section 3.1): `device_ids` is the row-major tensor of partition ids,
 * prod(shape) entries, a permutation of 0..P-1.  Host memory. */
typedef struct {
  int32_t rank;
  const int64_t* shape;
  const int64_t* device_ids;
} gspmd_mesh;

/* mesh_split(tensor, mesh, dims_mapping) of Section 3.1: dims_mapping[i] is the mesh
 * dimension tensor dimension i is split over, or -1.  Each mesh dimension at most once.
 * A tiled sharding given as a device tensor of the data's rank is the mesh whose
 * dimension i maps to data dimension i; a trailing replication dimension stays unmapped. */
typedef struct {
  int32_t rank;
  const int64_t* global_shape;   /* unpartitioned shape, host */
  const int32_t* dims_mapping;   /* host */
} gspmd_sharding;

/* Dot dimension numbers (Section 3.2): lhs_batch[i] pairs with rhs_batch[i] and
 * lhs_contract[i] with rhs_contract[i]; all other dimensions are non-contracting.
 * Output dimension order: batch, lhs non-contracting, rhs non-contracting. */
typedef struct {
  int32_t n_batch;
  const int32_t* lhs_batch;
  const int32_t* rhs_batch;
  int32_t n_contract;
  const int32_t* lhs_contract;
  const int32_t* rhs_contract;
} gspmd_dot_dims;

/* One partition's shard: device pointer to a row-major array of the static shard shape.
 * row_stride: distance in elements between consecutive indices of the second-to-last
 * dimension; 0 means dense (= static size of the last dimension).  Outer dimensions are
 * dense on top of it.  A row_stride that is a multiple of 8 elements together with a
 * 16-byte aligned pointer selects the fastest MFMA kernel for bf16 (an even row_stride with a 4-byte aligned pointer
 * its register-staged variant, see gspmd_kernel_path); an operand whose contiguous dimension
 * is contracted runs fastest when its rows start on 128-byte lines (row_stride a multiple of 64
 * elements: 9 % faster than a multiple of 8 that is not, at 8200 against 8256).  data may be NULL only for a
 * tensor with a zero-size dimension (no elements: nothing is read or written). */
typedef struct {
  void* data;          /* device */
  int32_t dtype;       /* gspmd_dtype */
  int64_t row_stride;  /* elements; 0 = dense */
} gspmd_shard_buf;

/* Utility (no counterpart in the paper): a short English name for a gspmd_status; never NULL. */
const char* gspmd_status_string(int32_t status);

/* Offset(S, d, i) of Section 3.5 with the static shard size of Section 4.1.
 * For partition `partition_id` and each tensor dimension i:
 *   shard_size[i] = ceil(D_i / n)          (n = size of the mapped mesh dimension, 1 if unmapped)
 *   offset[i]     = coord * shard_size[i]  (coord = the partition's position along that mesh dimension)
 *   valid_len[i]  = clamp(D_i - offset[i], 0, shard_size[i])
 * offset, valid_len: host arrays of sharding->rank entries; shard_size may be NULL.  Pure host work. */
int32_t gspmd_shard_bounds(const gspmd_mesh* mesh, const gspmd_sharding* sharding,
                           int64_t partition_id,
                           int64_t* offset, int64_t* valid_len, int64_t* shard_size);

/* Per mesh dimension, which communication-free case of the Dot it carries (Section 4.4);
 * GSPMD_ERR_NEEDS_RESHARD if any mesh dimension fits none (Section 4.5).
 * axis_class: host array of mesh->rank gspmd_axis_class values. */
int32_t gspmd_classify_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                           const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                           const gspmd_sharding* out_sh, int32_t* axis_class);

/* Output sharding of a Dot merged from the operand shardings (sharding propagation through Dot, Section 3.5):
 * an out dimension inherits the mesh dimension of the operand dimension it comes from, so that for every device
 * Offset(out, d, i) equals the operand's offset on every inherited sharded dimension; a mesh dimension that splits
 * a contracting pair leaves the output unsplit on it (a partial sum).  GSPMD_ERR_NEEDS_RESHARD if the operand
 * shardings are not compatible (a batch or contracting pair split differently on the two sides, one mesh dimension on
 * both a lhs and a rhs non-contracting dimension).  out_mapping / out_shape: host arrays of (n_batch + lhs free +
 * rhs free) entries, out_shape may be NULL; out_rank (nullable) receives the rank.  Pure host work. */
int32_t gspmd_infer_out_sharding(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                 const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                 int32_t* out_mapping, int64_t* out_shape, int32_t* out_rank);

/* Which index of a lowered GEMM's operand is the contiguous one; follows from where the Dot's contracting
 * dimensions sit in each operand.  0 = the forward einsums (lhs "...,c", rhs "c,..."). */
typedef enum {
  GSPMD_LAYOUT_LHS_K_MAJOR = 1,       /* lhs non-contracting dimension last:  A[m,k] at a_offset + k*lda + m */
  GSPMD_LAYOUT_RHS_K_CONTIGUOUS = 2   /* rhs contracting dimension last:      B[k,n] at b_offset + n*ldb + k */
} gspmd_layout_bits;

/* One strided GEMM of the list a partition's local Dot is lowered to:
 *   C[m, n] = sum_k A[m, k] * B[k, n]   for m < m_valid, n < n_valid, k < k_valid,   C = 0 on the rest of
 *   [m_static, n_static];  A[m,k] at lhs element a_offset + m*lda + k, B[k,n] at rhs element b_offset + k*ldb + n
 *   (the roles of the two indices exchanged where `layout` has the operand's gspmd_layout_bits bit set),
 *   C[m,n] at out element c_offset + m*ldc + n (offsets in elements from the shard buffers' data pointers). */
typedef struct {
  int64_t a_offset, b_offset, c_offset;
  int64_t lda, ldb, ldc;
  int32_t m_valid, n_valid, k_valid;
  int32_t m_static, n_static;
  int32_t layout;
  int32_t kernel;   /* gspmd_kernel_path of a launch made of such GEMMs, for bf16 operands at 16-byte aligned addresses */
  int32_t reserved;
} gspmd_gemm_desc;

/* Which contraction kernel the leading dimensions allow (the slowest one any GEMM of a launch needs is used for
 * the whole launch).  bf16 operands whose rows are not even 4-byte aligned, and fp32 operands, take the scalar kernel,
 * which is a correctness path many times slower than the other two. */
typedef enum {
  GSPMD_KERNEL_SCALAR = 0,       /* 64 x 64 tiles, fp32 FMA */
  GSPMD_KERNEL_MFMA_STAGED = 1,  /* MFMA, operand tiles through registers: lda and ldb even (rows 4-byte aligned) */
  GSPMD_KERNEL_MFMA = 2          /* MFMA, direct global->LDS loads: lda and ldb multiples of 8 elements */
} gspmd_kernel_path;

/* Utility for inspection and tests: the per-partition program of Section 4 made explicit.
 * How gspmd_local_dot lowers partition `partition_id`'s Dot (shard bounds -> flattened batch / free / contracting
 * extents -> one GEMM per batch entry and per index of a free dimension that padding keeps from flattening), without
 * touching the GPU.  *_row_stride as in gspmd_shard_buf: 0 = dense.  Writes min(count, capacity) descriptors to
 * `descs` (may be NULL when capacity is 0) and the total to `count`.  Pure host work; for inspection and tests. */
int32_t gspmd_plan_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                       const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh, const gspmd_sharding* out_sh,
                       int64_t lhs_row_stride, int64_t rhs_row_stride, int64_t out_row_stride,
                       int64_t partition_id, const int64_t* lhs_fill,
                       gspmd_gemm_desc* descs, int64_t capacity, int64_t* count);

/* Utility (the library allocates nothing, so the caller sizes the workspace):
 * bytes of device workspace gspmd_local_dot (partition_id >= 0) or gspmd_grouped_dot
 * (partition_id = -1: all partitions) needs for these arguments.  `has_fill` says whether a
 * fill-count array will be passed.  Pure host work. */
int32_t gspmd_dot_workspace_bytes(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                  const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                  const gspmd_sharding* out_sh, int64_t partition_id,
                                  int32_t has_fill, int64_t* bytes);

/* The local Dot of one partition (Section 4: the per-partition program of an Einsum whose
 * mesh dimensions are batch-, lhs-, rhs- or contracting-partitioned):
 *   out[b.., i.., j..] = sum_c lhs[b.., i.., c..] * rhs[b.., c.., j..]   over the partition's VALID extents,
 * fp32 accumulation, operands bf16 (out bf16 or f32) or f32 (out f32).
 * lhs/rhs/out: the partition's shard buffers (static shard shapes under lhs_sh/rhs_sh/out_sh).
 * Dimension order: the last dimension of each operand must be its innermost contracting or its
 * innermost non-contracting dimension, and the contracting dimensions must nest alike in both
 * operands (forward einsums "..c x c..", weight gradients "c.. x c..", input gradients
 * "..c x ..c" all qualify); anything else is GSPMD_ERR_UNSUPPORTED.
 * Positions >= valid length are masked to 0 in both operands along contracting dims and never
 * read along any dim (Section 4.1); out's padded region is written as 0.
 * If a mesh dimension is GSPMD_AXIS_CONTRACTING, out must be f32 and receives this
 * partition's partial sum (to be combined with gspmd_reduce_partials); `epilogue` must then be
 * GSPMD_EPILOGUE_NONE, and GSPMD_AXIS_CONTRACTING_SCATTER is GSPMD_ERR_UNSUPPORTED here (a slice of a
 * sum exists only after the exchange: use gspmd_grouped_dot).
 * epilogue: a gspmd_epilogue applied to every valid output element; padding stays 0.
 * lhs_fill (host, nullable): the number of occupied positions, per GLOBAL batch entry (row-major over the
 * global batch dims), of the first lhs dimension that is not a batch dimension -- the capacity slots of the
 * mixture-of-experts einsums (Section 5.4).  If that dimension is non-contracting it must be the only
 * non-contracting lhs dimension: rows at global position >= fill are masked and their out rows are 0.  If it
 * is contracting (the experts' weight gradient) it must be the outermost contracting dimension: positions
 * >= fill take no part in the sum in either operand.
 * workspace: device, 256-byte aligned, >= gspmd_dot_workspace_bytes(); contents are
 * overwritten and must stay untouched until the stream has run the call. */
int32_t gspmd_local_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                        const gspmd_shard_buf* lhs, const gspmd_sharding* lhs_sh,
                        const gspmd_shard_buf* rhs, const gspmd_sharding* rhs_sh,
                        const gspmd_shard_buf* out, const gspmd_sharding* out_sh,
                        int64_t partition_id, const int64_t* lhs_fill, int32_t epilogue,
                        void* workspace, int64_t workspace_bytes, void* hip_stream);

/* The local Dots of ALL partitions of the mesh in one ragged grouped launch
 * (single program, many partitions: Section 4).  lhs_shards/rhs_shards/out_shards: host
 * arrays of P entries indexed by partition id.  Partitions that hold the same data (they
 * differ only along mesh dimensions the tensor is not split on) may pass the same pointer.
 * If a mesh dimension is GSPMD_AXIS_CONTRACTING, fp32 partials go to the workspace and are
 * summed in ascending mesh-coordinate order into the out shard of every member of the reduce
 * group (the AllReduce of Section 4.2; members may share one buffer, written once); out may
 * then be bf16 or f32.  On a GSPMD_AXIS_CONTRACTING_SCATTER dimension every member receives only
 * its slice of the sum along the out dimension split there (ReduceScatter; the partials in the
 * workspace have that dimension whole).  `epilogue` is applied after the sum. */
int32_t gspmd_grouped_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                          const gspmd_shard_buf* lhs_shards, const gspmd_sharding* lhs_sh,
                          const gspmd_shard_buf* rhs_shards, const gspmd_sharding* rhs_sh,
                          const gspmd_shard_buf* out_shards, const gspmd_sharding* out_sh,
                          const int64_t* lhs_fill, int32_t epilogue,
                          void* workspace, int64_t workspace_bytes, void* hip_stream);

/* gspmd_grouped_dot for callers that cannot allocate device memory and so cannot provide a workspace (code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc): the same computation, with the launch
 * tables and the fp32 partials of a contracting split kept in a static device array of
 * GSPMD_NOALLOC_MAX_WORKSPACE_BYTES that the library holds on every GPU it is loaded on until the process ends.  Calls
 * nothing that allocates.  GSPMD_ERR_WORKSPACE if gspmd_dot_workspace_bytes(..., partition_id = -1) exceeds that size.
 * Every call on a GPU uses that GPU's one array (found on the current device at the first call there): calls that
 * overlap in time on one GPU -- different streams, different host threads -- race; the array keeps the last call's
 * contents, nothing in it needs to start out as zero.  Other arguments and results as gspmd_grouped_dot. */
#define GSPMD_NOALLOC_MAX_WORKSPACE_BYTES (32 * 1024 * 1024)
int32_t gspmd_grouped_dot_noalloc(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                  const gspmd_shard_buf* lhs_shards, const gspmd_sharding* lhs_sh,
                                  const gspmd_shard_buf* rhs_shards, const gspmd_sharding* rhs_sh,
                                  const gspmd_shard_buf* out_shards, const gspmd_sharding* out_sh,
                                  const int64_t* lhs_fill, int32_t epilogue, void* hip_stream);

/* out[i] = partials[0][i] + partials[1][i] + ... + partials[n_partials-1][i] in fp32, in that
 * order (the arithmetic of the AllReduce/ReduceScatter of Section 4.2 along a contracting
 * mesh dimension).  partials: host array of n_partials (1..16) device pointers to dense fp32
 * arrays of n_elems; out: device, f32 or bf16 (round-to-nearest-even), may alias partials[0]. */
int32_t gspmd_reduce_partials(const void* const* partials, int32_t n_partials, int64_t n_elems,
                              void* out, int32_t out_dtype, void* hip_stream);

/* Copy partition `partition_id`'s valid region of a dense global tensor (device) into its
 * shard buffer (the DynamicSlice of the appendix, Table 9); the shard's padded region is
 * filled with `pad_bits` (the element's bit pattern, low 16 bits for bf16; padding content is
 * arbitrary by Section 4.1, so tests poison it). */
int32_t gspmd_shard_extract(const gspmd_mesh* mesh, const gspmd_sharding* sharding,
                            int64_t partition_id, const void* global_data,
                            const gspmd_shard_buf* shard, uint32_t pad_bits, void* hip_stream);

/* Copy the valid region of a shard buffer to its place in a dense global tensor (device):
 * the DynamicUpdateSlice of the appendix, Table 9. */
int32_t gspmd_shard_assemble(const gspmd_mesh* mesh, const gspmd_sharding* sharding,
                             int64_t partition_id, const gspmd_shard_buf* shard,
                             void* global_data, void* hip_stream);

/* Utility: bytes of device workspace gspmd_reshard needs on this mesh.  Pure host work. */
int32_t gspmd_reshard_workspace_bytes(const gspmd_mesh* mesh, int64_t* bytes);

/* Resharding on the virtual mesh (Section 4.5): rewrite a tensor held under sharding `src_sh` into shard buffers under
 * `dst_sh`.  What would be an AllGather (a split dimension becomes whole), a DynamicSlice (a whole dimension becomes
 * split), an AllToAll (the split moves to another dimension or mesh dimension) or a CollectivePermute between real
 * devices is here one on-GPU gather: every element of every dst shard is read from the src shard that owns it (among
 * replicas, the one at the dst partition's own position along the mesh dimensions src is not split on).
 * src_shards / dst_shards: host arrays of P entries indexed by partition id, same dtype everywhere; all src shards
 * share one row_stride and so do all dst shards; partitions that hold the same data may pass the same pointer.  The
 * two shardings must have the same global shape.  Only valid positions of src shards are read; the padded part of
 * every dst shard is written as 0.  workspace: device, 256-byte aligned, >= gspmd_reshard_workspace_bytes(). */
int32_t gspmd_reshard(const gspmd_mesh* mesh,
                      const gspmd_sharding* src_sh, const gspmd_shard_buf* src_shards,
                      const gspmd_sharding* dst_sh, const gspmd_shard_buf* dst_shards,
                      void* workspace, int64_t workspace_bytes, void* hip_stream);

/* The operand shardings a Dot with output sharding `out_sh` can consume without communication, chosen as close to
 * the given ones as the output allows (the resharding decision of Section 4.5 for one Dot): per mesh dimension, an
 * operand dimension keeps its split if the output (or, for a contracting pair, the other operand) is split alike,
 * receives the split its out dimension has, and is made whole otherwise.  A mesh dimension that splits the same
 * contracting pair in both operands is kept (partial sums, possibly scattered).  lhs_mapping / rhs_mapping: host arrays
 * of lhs_sh->rank / rhs_sh->rank entries.  Shardings that are already compatible come back unchanged.  Pure host work. */
int32_t gspmd_compatible_operand_shardings(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                           const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                           const gspmd_sharding* out_sh,
                                           int32_t* lhs_mapping, int32_t* rhs_mapping);

/* Bytes of device workspace gspmd_resharded_dot needs (temporaries for the resharded operands of `in_dtype`, the tables
 * of the two reshards and the workspace of the grouped Dot).  Pure host work. */
int32_t gspmd_resharded_dot_workspace_bytes(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                                            const gspmd_sharding* lhs_sh, const gspmd_sharding* rhs_sh,
                                            const gspmd_sharding* out_sh, int32_t in_dtype, int64_t* bytes);

/* gspmd_grouped_dot for ANY operand shardings: operands whose sharding the Dot cannot consume as it is are first
 * rewritten (gspmd_reshard, into temporaries inside the workspace, rows padded to 8 elements) to the shardings
 * gspmd_compatible_operand_shardings names -- the AllGather / AllToAll / DynamicSlice a partitioner would insert in
 * front of the Dot (Section 4.5) -- then the grouped Dot runs on them; GSPMD_ERR_NEEDS_RESHARD is never returned.
 * Arguments as for gspmd_grouped_dot; lhs_fill counts refer to the global lhs as there. */
int32_t gspmd_resharded_dot(const gspmd_mesh* mesh, const gspmd_dot_dims* dims,
                            const gspmd_shard_buf* lhs_shards, const gspmd_sharding* lhs_sh,
                            const gspmd_shard_buf* rhs_shards, const gspmd_sharding* rhs_sh,
                            const gspmd_shard_buf* out_shards, const gspmd_sharding* out_sh,
                            const int64_t* lhs_fill, int32_t epilogue,
                            void* workspace, int64_t workspace_bytes, void* hip_stream);

/* Utility (no counterpart in the paper; a profiling aid for the MFMA contraction kernel).  While a record buffer is
 * set, every later Dot launch of this process (any entry point, any stream) makes workgroup b < n_records of its
 * MFMA kernel write record b: eight 64-bit words of the GPU's 100 MHz constant-rate counter at kernel entry (bits
 * 52-63 hold XCD id << 8 | compute-unit id bits), tile decoded, first tile loads issued, K loop entered, K loop left,
 * epilogue entered, stores issued, stores complete; a workgroup that leaves early (a joined contribution that is not
 * the last to arrive) leaves words 5 to 7 untouched.  device_records: device memory of n_records * 64 bytes, 8-byte
 * aligned, owned by the caller, who clears it and keeps it alive until the launches have finished;
 * NULL or n_records 0 switches the timeline off (the default; the kernel then skips the stamps on one uniform branch).
 * The setting is process-wide, not per stream: launches that overlap write to the same records, and a launch recorded
 * into a HIP graph keeps the buffer it was recorded with.  Results of the Dot are unchanged.  Returns GSPMD_ERR_BAD_BUFFER for a misaligned pointer or a count outside [0, 2^31). */
int32_t gspmd_set_tile_timeline(void* device_records, int64_t n_records);

#ifdef __cplusplus
}
#endif
#endif /* GSPMD_H_ */
