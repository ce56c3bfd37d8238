/*
 * tpx - re-partitioning of a training job's state between two multi-dimensional
 * parallelism configurations, on one MI355X (gfx950).
 *
 * The job state is a parallelizable tensor collection PTC = (T, sigma, phi, alpha)
 * (paper section 4.1, equation 1): state tensors T, a slicing function sigma
 * (tensor parallelism), a partitioning function phi (pipeline stages and
 * data-parallel replicas) and an allocation function alpha (sub-collection ->
 * device).  Given the current PTC and a new PTC' over the same tensors, a
 * reconfiguration plan made of split, re-partition (move) and merge operations
 * turns the state of the one into the state of the other (section 4.2,
 * algorithm 1), and a state transformer applies it (section 5.1, step 4).
 *
 * Here every "device" of either configuration is one flat buffer in the HBM of a
 * single GPU: rank (t, p, d) of a configuration (T, P, D) is buffer index
 * t + T*(d + D*p).  tpx_plan() computes the plan on the host; tpx_execute()
 * applies the whole plan with one kernel launch.
 *
 * Conventions for every call
 *   - pointers are HOST pointers unless the comment says DEVICE;
 *   - the caller owns all device memory (rank buffers and the workspace); the
 *     library owns only the host-side plan object, released by tpx_free();
 *   - a call returns TPX_OK or a negative tpx_status, never throws or aborts;
 *     out-parameters are untouched on error; tpx_last_error() returns a
 *     thread-local description of the last failure on the calling thread.
 *
 * Limits: TPX_MAX_RANKS buffers per side; 2^31 tiles per plan (at the default
 * 64 KiB per tile far more than one GPU's memory holds); a move may be as long
 * as a buffer, except that a move between different storage orders may not
 * exceed 2^32 - 1 elements along either axis of the plane it transposes.  A
 * plan beyond these is refused with INVALID_ARG.
 */
#ifndef TPX_H
#define TPX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tpx_plan_s tpx_plan_t; /* opaque */

typedef enum {
  TPX_OK = 0,
  TPX_ERR_INVALID_ARG = -1,   /* NULL pointer, zero degree, unsupported size, bad index */
  TPX_ERR_INDIVISIBLE = -2,   /* heads / hidden / ffn / vocabulary / layers / batch not divisible */
  TPX_ERR_BAD_STAGE_MAP = -3, /* stage boundaries not ascending from 0 to n_layers */
  TPX_ERR_OOM = -4,           /* host allocation failed */
  TPX_ERR_HIP = -5,           /* a HIP runtime call failed (message has the HIP error) */
  TPX_ERR_MISALIGNED = -6,    /* a device pointer is not aligned as the call requires */
  TPX_ERR_CURSOR = -7,        /* dataset cursors are not those of a whole number of steps */
  TPX_ERR_UNRECOVERABLE = -8, /* some state has no surviving source holder */
  TPX_ERR_STALE_WORKSPACE = -9, /* the workspace does not (or no longer) hold this plan's tables */
  TPX_ERR_TOO_LARGE = -10     /* the plan tables do not fit the static table array of tpx_execute_static */
} tpx_status;

#define TPX_MAX_RANKS 128u    /* buffers per side */
#define TPX_SIDE_SRC 0
#define TPX_SIDE_DST 1

/* ---- the tensor collection T: a GPT-style model and its state mix ------------------- */
#define TPX_MODEL_TIED_HEAD 1u /* last stage also holds the word embeddings when P > 1 */

typedef struct {
  uint32_t n_layers, hidden, n_heads, ffn, vocab_true, max_pos;
  uint32_t vocab_divisor;       /* 0: vocab_true must divide by T; else rows are padded to a multiple of divisor*T */
  uint32_t n_state_kinds;       /* 1..4 state tensors per parameter (weight, master copy, Adam m, Adam v, ...) */
  uint8_t  state_elem_bytes[4]; /* element size of each state kind: 1, 2, 4 or 8 */
  uint32_t flags;               /* TPX_MODEL_* */
} tpx_model;

/* ---- sigma, phi, alpha of one configuration ------------------------------------------ */
typedef struct {
  uint32_t T, P, D;                  /* tensor-, pipeline-, data-parallel degree */
  const uint32_t* stage_first_layer; /* phi: P+1 ascending layer boundaries, [0]=0, [P]=n_layers; NULL = n_layers/P each */
  uint32_t qkv_layout;               /* sigma of the fused QKV tensors: 0 head-major [a,3,d,*], 1 qkv-major [3,a,d,*] */
  uint32_t w_transposed;             /* 1: 2-D weights are stored [in, out] instead of [out, in] */
  const uint8_t* rank_alive;         /* T*P*D bytes or NULL (= all 1).  Source configuration: 0 = this rank's buffer is
                                        lost (section 5.3) and is never read.  Destination configuration: 0 = this rank
                                        is not to be built (say, it survived and keeps its state): no move is planned
                                        for it, its buffer is never written and may be NULL in tpx_execute. */
  const uint32_t* layer_stage;       /* phi as an arbitrary map: n_layers stage indices (< P), e.g. the interleaved chunks
                                        of a virtual pipeline; overrides stage_first_layer; NULL = not used.  A stage
                                        holds its layers in ascending order; embeddings stay on stage 0, the final
                                        LayerNorm on stage P-1. */
  uint32_t shard_kinds;              /* phi, sharded data parallelism: bit k set = state kind k is not replicated over
                                        the D replicas but cut between them: of each block its (t, p) share holds,
                                        replica d stores chunk d of ceil(n / D) rows along the block's outermost
                                        stored axis (n its extent there); short or empty chunks at the end; a
                                        replica with an empty chunk has no entry for the tensor.  0 = none. */
} tpx_parallel;

/* One stored sub-tensor of a rank buffer ("/<rank>/<module path>/<param>", section 5.2).
 * The full tensor has `ndim` canonical axes; the block covers [lo, hi) on each and is stored
 * dense row-major with stored axis i = canonical axis perm[i]. */
typedef struct {
  uint32_t tensor_id;  /* 0 word emb, 1 pos emb, 2/3 final LayerNorm w/b, 4 + 12*layer + k for the k-th per-layer tensor */
  uint32_t kind;       /* state kind index */
  uint32_t elem_bytes;
  uint32_t ndim;
  uint32_t name;       /* index into the 16 parameter names, see tpx_param_name() */
  int32_t  layer;      /* -1 for global tensors */
  uint64_t offset;     /* byte offset inside the rank buffer, multiple of 256 */
  uint64_t nbytes;
  uint64_t full_shape[4], lo[4], hi[4];
  uint32_t perm[4];
} tpx_entry;

/* One move of the plan (algorithm 1: move(w, r_w, r') together with the split that produced w
 * and w's place in the merge).  Byte j of unit (i_0, .., i_{ndim-1}), 0 <= i_k < extent[k],
 * 0 <= j < run_bytes, goes from  src_off + sum_k i_k*src_stride[k] + j  of buffer src_rank
 * to  dst_off + sum_k i_k*dst_stride[k] + j  of buffer dst_rank.  TPX_BOX_FILL writes zeros and has
 * no source.  TPX_BOX_TRANSPOSE moves single elements (run_bytes == elem_bytes): no axis is
 * contiguous on both sides.  Axes are ordered by descending destination stride. */
#define TPX_BOX_COPY 0u
#define TPX_BOX_FILL 1u
#define TPX_BOX_TRANSPOSE 2u
typedef struct {
  uint32_t kind;
  uint32_t src_rank, dst_rank;
  uint32_t n_dst;           /* multicast: the same bytes also go, at the same offsets, to buffers          */
  uint32_t dst_rank_stride; /* dst_rank + k*dst_rank_stride, k < n_dst (data-parallel replicas); n_dst >= 1 */
  uint32_t ndim;          /* number of outer axes used, 0..4 */
  uint32_t elem_bytes;
  uint32_t tensor_id;     /* of the first tensor it covers (boxes of neighbouring tensors may be merged) */
  uint64_t src_off, dst_off;
  uint64_t run_bytes;
  uint64_t extent[4];
  uint64_t src_stride[4]; /* bytes */
  uint64_t dst_stride[4]; /* bytes */
} tpx_box;

/* One unit of GPU work: a bounded piece of one box, executed by one workgroup.  Tiles are not stored:
 * the kernel (and tpx_get_tile, with the same code) derives tile number b from a compact box table.
 * Unit (i, j), 0 <= i < nrows, 0 <= j < run_units, of
 * 1 << unit_log2 bytes goes from  src_off + i*src_pitch + j*src_step  to
 * dst_off + i*dst_pitch + j*dst_step. */
#define TPX_TILE_COPY 0u      /* src_step == dst_step == unit: rows are contiguous on both sides */
#define TPX_TILE_FILL 1u      /* like COPY, zeros instead of a source */
#define TPX_TILE_TRANSPOSE 2u /* unit = element; rows are contiguous on the source (src_step == unit),
                                 columns on the destination (dst_pitch == unit); staged through LDS */
#define TPX_TILE_GATHER 3u    /* unit = element; arbitrary steps (degenerate transposes) */
#define TPX_TILE_MERGE 4u     /* the merge of algorithm 1 done inside the tile: destination rows are written whole;
                                 every row is the concatenation of n_seg column blocks, block k coming from
                                 segment seg_first + k (its own source buffer, offset, row pitch and width);
                                 seg_units = the common width of the blocks in units, or 0 when they differ
                                 (then see tpx_segment.units); src_off / src_pitch / src_rank are unused,
                                 src_off = first row of the tile within the box (add src_off * segment pitch
                                 to the segment's offset) */
#define TPX_TILE_PACK 5u      /* several short contiguous moves into the same destination buffer(s), done by one
                                 workgroup so that none of them occupies a compute unit by itself: the tile is ONE
                                 row of run_units 16-byte units, the concatenation of segments seg_first ..
                                 seg_first + n_seg - 1; each segment has its own source (buffer, offset), its own
                                 place in the destination buffer(s) (tpx_segment.dst_off) and its own length;
                                 the tile's src_off, dst_off, pitches and src_rank are 0 and unused */
typedef struct {
  uint64_t src_off, dst_off;  /* bytes, inside the rank buffers */
  uint64_t src_pitch, dst_pitch;
  uint64_t src_step, dst_step;
  uint32_t run_units;
  uint32_t nrows;
  uint16_t src_rank, dst_rank;
  uint8_t  kind;
  uint8_t  unit_log2;         /* 4 (16-byte vectors) when offsets, pitches and run length allow, else smaller */
  uint8_t  n_dst;             /* written to buffers dst_rank + k*dst_rank_stride, k < n_dst */
  uint8_t  dst_rank_stride;
  uint32_t seg_first;         /* MERGE and PACK tiles: first segment, number of segments, units per segment (MERGE) */
  uint32_t n_seg;
  uint32_t seg_units;
  uint32_t pad_;
} tpx_tile;

/* One source of a MERGE tile (the rows of a source sub-tensor piece) or one move of a PACK tile. */
typedef struct {
  uint64_t src_off;           /* MERGE: byte offset of row 0 of the box in buffer src_rank; PACK: of the move's first byte */
  uint64_t src_pitch;         /* MERGE: bytes between rows; PACK: index of the segment's first unit within the tile */
  uint32_t src_rank;
  uint32_t units;             /* MERGE: width of the column block it contributes; PACK: length; in 16-byte units */
  uint64_t dst_off;           /* PACK: byte offset of the move in the destination buffer(s); MERGE: 0 */
} tpx_segment;

typedef struct {
  uint64_t n_pieces;          /* sub-tensor pieces produced by the split step */
  uint64_t n_boxes;           /* moves after merging neighbours */
  uint64_t n_tiles;
  uint64_t bytes_read;        /* source bytes read; a move replicated to several destinations reads once */
  uint64_t bytes_written;     /* destination bytes written (= all destination tensor bytes) */
  uint64_t bytes_fill;        /* zero-filled destination bytes (vocabulary padding growth) */
  uint64_t bytes_cross_rank;  /* bytes whose source buffer index differs from the destination's */
  uint64_t plan_ns;           /* host time spent in tpx_plan */
} tpx_stats_t;

/* Options of one plan; NULL wherever a tpx_plan_opts* is taken means all defaults (a zero field too).
 *   tile_bytes     upper bound of bytes per tile, the unit of GPU work: a power of two, 4096 .. 4194304; default
 *                  65536.  Small jobs use smaller tiles, down to 16384, so that the launch still has thousands of
 *                  workgroups; a plan with transposing moves never uses larger ones.
 *   max_multicast  most replicas one move may be written to (1 .. 128; default 8; 1 = every replica is copied
 *                  separately).
 *   share_reads    0 (default): every destination rank reads from the holder section 6.5's locality rule picks for
 *                  it (its own device first), which minimises bytes_cross_rank; 1: all ranks of a replica group
 *                  read what the group's first rank reads, so a piece wanted by n replicas is read once and written
 *                  n times - fewer bytes through memory when all buffers share one GPU.
 *   pack_bytes     contiguous, 16-byte aligned moves of at most this many bytes do not get a tile each: up to 64 of
 *                  them that go to the same destination buffer(s) share one PACK tile.  0 = default (a quarter of
 *                  the tile size in use); 1 = pack nothing; at most tile_bytes. */
typedef struct {
  uint64_t tile_bytes;
  uint32_t max_multicast;
  uint32_t share_reads;
  uint32_t pack_bytes;
  uint32_t reserved_;         /* 0 */
} tpx_plan_opts;

/* Plan the transformation of the model state of `model` from configuration src to dst (section 4.2,
 * algorithm 1: split, re-partition, merge).  Host only; all arguments are HOST pointers read during the
 * call (nothing is retained).  On success *out owns the plan until tpx_free().  The plan fixes the layout
 * of every rank buffer of both sides (tpx_buffer_bytes, tpx_manifest): rank (t, p, d) is buffer
 * t + T*(d + D*p); inside it one arena per state kind, each holding the stage's tensors in the order
 * embeddings, layers ascending (12 tensors each), final LayerNorm, 256-byte aligned.
 * Errors: INVALID_ARG (NULL, zero degree, > TPX_MAX_RANKS ranks, element size not 1/2/4/8, option out of
 * range), INDIVISIBLE, BAD_STAGE_MAP, UNRECOVERABLE (src->rank_alive leaves a tensor without holder), OOM. */
tpx_status tpx_plan(const tpx_model* model, const tpx_parallel* src, const tpx_parallel* dst,
                    const tpx_plan_opts* opts, tpx_plan_t** out);

/* A parallelizable tensor collection given explicitly (section 4.1, equation 1; section 5.1: the per-GPU
 * description a model parallelizer hands over): for every rank, the sub-tensors it stores.  sigma is the
 * set of boxes [lo, hi) of each tensor, phi and alpha are "which rank's list an entry is in" and its
 * offset.  Anything expressible this way can be re-partitioned: tensor, pipeline and data parallelism,
 * expert parallelism (phi groups whole expert tensors), sequence parallelism (sigma slices sample
 * tensors), sharded optimizer state (section 4.3).  Used fields of tpx_entry: tensor_id and kind (together
 * the identity of a state tensor), elem_bytes (1, 2, 4, 8), ndim (1..4), offset, full_shape, lo, hi, perm;
 * nbytes may be 0 (computed); name and layer are not interpreted.  An offset of TPX_OFFSET_AUTO asks the
 * library to place the entry itself: a rank's entries are then packed in list order, each at the next
 * 256-byte boundary after the entry before it (tpx_manifest tells where); a rank's entries must all be
 * placed that way or none. */
#define TPX_OFFSET_AUTO UINT64_MAX
typedef struct {
  uint32_t n_ranks;                 /* 1..TPX_MAX_RANKS */
  const uint32_t* n_entries;        /* n_ranks counts */
  const tpx_entry* const* entries;  /* n_ranks arrays */
  const uint64_t* rank_bytes;       /* n_ranks buffer sizes, or NULL: end of the last sub-tensor rounded up to 256 */
  const uint8_t* rank_alive;        /* n_ranks flags or NULL: source 0 = lost, destination 0 = not to be built
                                       (as in tpx_parallel) */
} tpx_ptc;

/* Plan the transformation of PTC src into PTC dst over the same tensors (algorithm 1).  Within one side the
 * sub-tensors of a tensor must be equal (replicas) or disjoint; the source's must tile every destination
 * sub-tensor, except rows of axis 0 beyond the source tensor's extent, which are zero-filled.  Destination
 * ranks with identical manifests whose indices form an arithmetic progression are treated as replicas
 * (multicast moves).  Errors: INVALID_ARG (malformed entry, overlap, missing tensor, no tiling),
 * UNRECOVERABLE, OOM. */
tpx_status tpx_plan_ptc(const tpx_ptc* src, const tpx_ptc* dst, const tpx_plan_opts* opts, tpx_plan_t** out);

/* A range query on a stored collection (section 5.2: "/2/embedding/weight[:, 2:4]" selects [2, 4) on axis 1):
 * the box [lo, hi) of state tensor (tensor_id, kind), in the full tensor's coordinates. */
typedef struct {
  uint32_t tensor_id, kind;
  uint64_t lo[4], hi[4];
} tpx_query;

/* Plan the gathering of n_queries boxes of the collection src, from whichever ranks hold their pieces, into
 * ONE destination buffer: box i is stored dense, row-major in the tensor's own axis order, at the next
 * 256-byte boundary after box i-1 (tpx_manifest(plan, TPX_SIDE_DST, 0, i) gives its place,
 * tpx_buffer_bytes(plan, TPX_SIDE_DST, 0) the size to allocate).  Element size and rank of each tensor are
 * taken from src.  It is tpx_plan_ptc with a one-rank destination the library lays out.
 * Errors: INVALID_ARG (a tensor that src does not have, lo >= hi, hi beyond the tensor), UNRECOVERABLE, OOM. */
tpx_status tpx_plan_query(const tpx_ptc* src, uint32_t n_queries, const tpx_query* queries,
                          const tpx_plan_opts* opts, tpx_plan_t** out);

/* Plan the transformation of the dataset state (sections 2.2 and 5.2): per-replica sample-index arrays
 * of one epoch are re-partitioned from D_src to D_dst replicas with the global batch unchanged, so that
 * the job consumes the same samples in the same order.  Replica j's index array holds, for every step k,
 * entries [k*B + j*b, k*B + (j+1)*b) of the global order (b = B/D), clipped to n_samples; buffer j of a
 * side is that array (index_elem_bytes per entry: 8 for sample ids, 16 for (offset, length) pairs).
 * src_cursors[j] = consumed entries of source partition j; dst_cursors (D_dst entries, written on success)
 * receives the equivalent positions.  Errors: INVALID_ARG, INDIVISIBLE (B % D), CURSOR. */
tpx_status tpx_plan_dataset(uint64_t n_samples, uint32_t global_batch, uint32_t index_elem_bytes,
                            uint32_t D_src, uint32_t D_dst, const uint64_t* src_cursors,
                            uint64_t* dst_cursors, const tpx_plan_opts* opts, tpx_plan_t** out);

/* Queries (cheap, host only; the plan is not modified and nothing is allocated for the caller).
 * side: TPX_SIDE_SRC / TPX_SIDE_DST.  Out-of-range indices give 0 / INVALID_ARG.  tpx_manifest lists the
 * sub-tensors of a rank buffer (section 5.2's tree of a state partition, flattened); tpx_get_box the moves
 * of the plan; tpx_get_tile / tpx_get_segment what workgroup-sized unit of work number i does, computed by
 * the code the kernel itself uses.  Dataset plans have buffers but no manifest entries. */
uint32_t   tpx_num_buffers(const tpx_plan_t*, int side);
uint64_t   tpx_buffer_bytes(const tpx_plan_t*, int side, uint32_t rank);
uint32_t   tpx_num_entries(const tpx_plan_t*, int side, uint32_t rank);
tpx_status tpx_manifest(const tpx_plan_t*, int side, uint32_t rank, uint32_t i, tpx_entry* out);
const char* tpx_param_name(uint32_t name); /* static string, NULL if out of range */
tpx_status tpx_stats(const tpx_plan_t*, tpx_stats_t* out);
uint64_t   tpx_num_boxes(const tpx_plan_t*);
tpx_status tpx_get_box(const tpx_plan_t*, uint64_t i, tpx_box* out);
uint64_t   tpx_num_tiles(const tpx_plan_t*);
tpx_status tpx_get_tile(const tpx_plan_t*, uint64_t i, tpx_tile* out);
uint64_t   tpx_num_segments(const tpx_plan_t*);
tpx_status tpx_get_segment(const tpx_plan_t*, uint64_t i, tpx_segment* out);

/* Traffic matrix of the plan: out[i * n_dst + j] = bytes that destination rank j receives from source rank i
 * (n_src x n_dst entries, row-major; a move replicated to several destinations counts once per destination;
 * zero fill has no source and is not counted).  With one device per rank this is the exchange the locality
 * rule of section 6.5 minimises: the diagonal (i == j) stays on the device, the rest crosses devices
 * (its sum is tpx_stats.bytes_cross_rank).  `out` is a HOST array of tpx_num_buffers(src) * tpx_num_buffers(dst)
 * entries.  Errors: INVALID_ARG. */
tpx_status tpx_traffic(const tpx_plan_t*, uint64_t* out);

/* DEVICE bytes tpx_execute needs in `workspace` (a header, then the plan tables: flat boxes, tile prefix
 * sums, the segments of merge and pack tiles). */
uint64_t   tpx_workspace_bytes(const tpx_plan_t*);

/* Apply the plan (section 5.1, step 4): one kernel launch on `hip_stream` (a hipStream_t, NULL = the
 * default stream).  src_bufs / dst_bufs are HOST arrays of DEVICE pointers, one per rank of the side,
 * each at least tpx_buffer_bytes() long and 16-byte aligned (256 recommended); entries of lost source
 * ranks and of destination ranks that are not built (rank_alive) may be NULL.  workspace is a DEVICE pointer
 * to tpx_workspace_bytes() bytes, 64-byte aligned.  Every tensor byte of every destination rank that is
 * built is written exactly once; bytes between tensors are left untouched; sources are only read and must
 * not overlap destinations.  The call does not wait for the kernel.
 * The library remembers, per workspace address, which plan's tables it last copied there.  When that is not
 * this plan (first use, or another plan has used the workspace since), the call copies the tables on
 * `hip_stream` and waits for the copy; otherwise it only launches.  So two plans may take turns on one
 * workspace, and any number of threads may execute one plan (the plan is not modified).  What the library
 * cannot see is the caller overwriting or freeing the workspace: tell it with tpx_workspace_forget().
 * Should the tables be overwritten unnoticed, the launch moves nothing (see tpx_workspace_check()).
 * Errors: INVALID_ARG (NULL where a pointer is needed), MISALIGNED (a rank buffer not 16-byte aligned, the
 * workspace not 64-byte aligned), HIP. */
tpx_status tpx_execute(const tpx_plan_t*, const void* const* src_bufs, void* const* dst_bufs,
                       void* workspace, void* hip_stream);

/* tpx_execute for callers that cannot allocate device memory and so have no workspace to hand over: code
 * whose launches are recorded into a HIP graph by someone else, tight serving loops, harnesses that forbid
 * hipMalloc.  The plan tables live in a static device array inside the library instead, one array of
 * TPX_STATIC_WORKSPACE_BYTES per GPU, held until the process ends; its address on the current device is
 * looked up on the first call there.  The call allocates nothing on the device or through any library
 * routine, takes the same src_bufs / dst_bufs (HOST arrays of DEVICE pointers, same alignment and NULL
 * rules), launches the same kernel on `hip_stream` (which must belong to the current device) and gives the
 * same bytes as tpx_execute.  When the array does not hold this plan's tables already (first call, or
 * another plan ran in between), they are copied there on `hip_stream` and the call waits for that copy;
 * otherwise it only launches.  All calls on one GPU share that GPU's array: calls that overlap there (other
 * threads, or other streams while an earlier launch of a different plan is still running) race on it;
 * calls on one stream, or separated by a wait, do not.  The plan is not modified.
 * Errors: TOO_LARGE (tpx_workspace_bytes() > TPX_STATIC_WORKSPACE_BYTES: use tpx_execute), INVALID_ARG,
 * MISALIGNED, HIP. */
#define TPX_STATIC_WORKSPACE_BYTES (4u << 20)
tpx_status tpx_execute_static(const tpx_plan_t*, const void* const* src_bufs, void* const* dst_bufs, void* hip_stream);

/* Optional: copy the plan tables into `workspace` now (and wait for the copy), so that a following
 * tpx_execute with the same workspace only launches the kernel.  Required before a tpx_execute that is
 * recorded into a HIP graph (stream capture allows neither the wait nor a copy from pageable host memory):
 * prepare outside the capture, then capture the execute, which is then a single kernel node.
 * Errors: INVALID_ARG, MISALIGNED, HIP. */
tpx_status tpx_prepare(const tpx_plan_t*, void* workspace, void* hip_stream);

/* Forget what the library believes about `workspace` (call after overwriting or freeing it): the next
 * tpx_execute or tpx_prepare with that address copies the tables again.  NULL forgets every workspace. */
void tpx_workspace_forget(const void* workspace);

/* The tables start with a header stamped with an id unique to the plan, and the kernel compares it with
 * the plan it was launched for: a tpx_execute on a workspace that another plan's tables (or anything
 * else) have overwritten since the upload moves nothing instead of following foreign tables.  This call
 * tells the caller about it: it waits for `hip_stream`, reads the header back and returns
 * TPX_ERR_STALE_WORKSPACE unless it is this plan's (and then also forgets the workspace, so that the next
 * execute copies the tables again).  Use it after tpx_execute when the workspace's history is in doubt.
 * Errors: INVALID_ARG, HIP, STALE_WORKSPACE. */
tpx_status tpx_workspace_check(const tpx_plan_t*, const void* workspace, void* hip_stream);

/* Release a plan (NULL is allowed).  The caller must make sure no tpx_execute launch of it is still being
 * issued; kernels already launched do not need the host plan. */
void tpx_free(tpx_plan_t*);

/* Description of the last failure on the calling thread (never NULL; valid until that thread's next failure). */
const char* tpx_last_error(void);

/* Process-wide knobs of the executor, for experiments with the kernel (each is read and written atomically by
 * any thread; what a plan contains never depends on them):
 *   "variant"     kernel variant, 0 (default) = chosen from the tile size: 512 threads per workgroup with eight
 *                 nontemporal 16-byte loads in flight per thread for 64 KiB tiles, 1024 threads for tiles of 128 KiB
 *                 and more, 256 threads x 4 loads for smaller tiles; other values are a bit field documented in the
 *                 kernel source
 *   "streams"     tile order (1 .. 1024; default 4): the tile sequence is cut into `streams` contiguous parts that
 *                 advance side by side, so concurrent workgroups touch `streams` distant regions of the buffers
 *   "chunk"       tile order (0 .. 4096; default 0 = automatic: 8, or 1 for plans with transposing moves): within a
 *                 stream, each of the GPU's 8 XCDs takes `chunk` consecutive tiles at a time (used when `streams`
 *                 divides 8); 1 = workgroup b takes the (b / streams)-th tile of stream b % streams
 *   "occupancy"   workgroups per CU, enforced through the LDS size a workgroup requests (0 .. 16; default 0 =
 *                 automatic: one for 512-thread workgroups, unconstrained otherwise)
 * Errors: INVALID_ARG for an unknown key or a value out of range. */
tpx_status tpx_set_option(const char* key, uint64_t value);

/* Plain device-to-device copy of nbytes (multiple of 16, DEVICE pointers 16-byte aligned) by a simple
 * grid-stride kernel on hip_stream: the yardstick for achievable HBM copy bandwidth and the
 * calibration point for hardware traffic counters.  Errors: INVALID_ARG, MISALIGNED, HIP. */
tpx_status tpx_probe_copy(void* dst, const void* src, uint64_t nbytes, void* hip_stream);

/* Read-only and write-only yardsticks: what the memory gives a pure read stream and a pure write stream in the
 * launch shape and tile order of tpx_execute's default copy tile (which is within 1 % of the best write-only and
 * within 3 % of the best read-only launch found); a copy has to retire both kinds.
 * tpx_probe_read reads nbytes (multiple of 16) from DEVICE src; `sink` is 16 DEVICE bytes the kernel may write
 * (it does so only when the words a thread read XOR to one particular value: that dependency is what keeps the
 * reads from being optimised away).  tpx_probe_fill writes the 32-bit `value` over nbytes of DEVICE dst.
 * Asynchronous on hip_stream.  Errors: INVALID_ARG, MISALIGNED, HIP. */
tpx_status tpx_probe_read(const void* src, uint64_t nbytes, void* sink, void* hip_stream);
tpx_status tpx_probe_fill(void* dst, uint64_t nbytes, uint32_t value, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TPX_H */
