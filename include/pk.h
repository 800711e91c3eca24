/* pk — packed multi-field embedding layer for one MI355X (gfx950).
 *
 * C ABI of the library.  The operations are those of the embedding layer of a
 * wide-and-deep recommender model as the paper states them:
 *   - Sec. II-D: Unique (drop repeated IDs), Gather (fetch embedding rows),
 *     SegmentReduction (pool rows per sample), backward pass = mirror image;
 *   - Sec. III-B (D-Packing / K-Packing, Fig. 7): the ID tensors of all fields
 *     whose tables share an embedding dimension are combined into one packed
 *     ID tensor and handled by one packed operation, and memory-bound steps
 *     are fused with each other;
 *   - the sparse Adagrad update is fixed by the workload configurations, not
 *     by the paper.
 *
 * Conventions
 *   - Every pointer says "host" or "device".  The library owns only the
 *     host-side plan (plus a few KB of device metadata it uploads on the first
 *     call that uses a plan).  Tables, accumulators, inputs, outputs and the
 *     workspace are allocated and freed by the caller.
 *   - pk_forward / pk_backward_update only enqueue work on the given HIP
 *     stream and return; they never synchronise.  Data-dependent sizes (number
 *     of distinct keys) stay in device memory.
 *   - All functions return a pk_status (0 = success) and never throw;
 *     pk_last_error() gives a thread-local message for the last failure.
 *   - Limits: total rows of a pack < 2^32, of a table <= 2^30; dim <= 256; nnz < 2^31;
 *     B * out_dim < 2^32; at most 4096 fields and 4096 tables.
 */
#ifndef PK_H
#define PK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PK_OK = 0,
    PK_EINVAL = 1,      /* null pointer, bad enum, non-positive size            */
    PK_ESHAPE = 2,      /* B / nnz / stride inconsistent with the plan          */
    PK_EWORKSPACE = 3,  /* workspace too small or misaligned                    */
    PK_EOVERFLOW = 4,   /* a documented limit would be exceeded                 */
    PK_EHIP = 5,        /* a HIP call failed                                    */
    PK_ENOMEM = 6       /* host allocation failed                               */
} pk_status;

typedef enum { PK_F32 = 0, PK_BF16 = 1 } pk_dtype;
typedef enum { PK_SUM = 0, PK_MEAN = 1 } pk_pool;

/* One embedding table: rows x dim elements of dtype. */
typedef struct { int64_t rows; int32_t dim; int32_t dtype; } pk_table_desc;
/* One feature field: the table it reads (several fields may share a table)
 * and how its bag of rows is pooled (Sec. II-D SegmentReduction; mean divides
 * by the bag length counting repeats; an empty bag pools to zeros). */
typedef struct { int32_t table; int32_t pool; } pk_field_desc;

typedef struct {
    int32_t max_batch;   /* largest B that will be passed (0 = no limit checked)   */
    int64_t max_nnz;     /* largest nnz that will be passed (0 = no limit checked) */
    int32_t max_shards;  /* Eq. 1 shard split of heavy packs; 0 or 1 = off          */
    const double* field_volume; /* host, [n_fields] or NULL: occurrences per field
                                   from warm-up statistics, used by the Eq. 1 split */
    int32_t interleave_groups;  /* Sec. III-C K-Interleaving: the packs are dealt to this
                                   many groups (pack p -> group p mod G); a group's packed
                                   operations run one after another, the groups side by
                                   side (one internal HIP stream each, joined before the
                                   call's work on hip_stream is complete).  0 = chosen by
                                   batch size, 1 = none, at most 8.  Results do not depend
                                   on it.                                               */
    int32_t debug;              /* for tests and measurements; results do not depend on it.
                                   bit 0: no internal streams, every kernel on hip_stream;
                                   bit 1: the partitioned dedup also for small batches      */
} pk_plan_opts;

typedef struct pk_plan pk_plan;   /* opaque, host memory, owned by the library */

/* ---- plan (Sec. III-B: pack fields whose tables share the dimension) --------
 * Packs are the distinct (dim, dtype) pairs in ascending (dim, dtype) order.
 * With opts->max_shards > 1 the heavy ones are split (Sec. III-B, Eq. 1): the
 * volume of a pack is the number of floats it gathers, sum over its tables of
 * dim x occurrences (occurrences of a table = sum of field_volume over the
 * fields that read it; every field counts 1 when field_volume is NULL); a pack
 * whose volume is above the average over the packs gets round(volume / smallest
 * non-zero volume) shards, at most max_shards and at most one per table, and
 * its tables are dealt to the shards in turn (the paper's example: one
 * operation for dim 8, four shards for dim 32).  Shards
 * are packs of their own, ordered (dim, dtype, shard).
 * Inside a pack the tables are stacked in table-index order into ONE caller
 * buffer [total_rows, dim]; pk_plan_table_slot tells where each table starts.
 * Fields of a pack are numbered (slots) in field-index order.  The pooled
 * outputs of one sample are concatenated in field order: field f occupies
 * columns [col(f), col(f)+dim) of out[B, out_dim].
 * tables, fields, opts: host.  *out receives the plan on success. */
pk_status pk_plan_create(const pk_table_desc* tables, int32_t n_tables,
                         const pk_field_desc* fields, int32_t n_fields,
                         const pk_plan_opts* opts, pk_plan** out);
void      pk_plan_destroy(pk_plan* plan);
int32_t   pk_plan_num_packs(const pk_plan* plan);
/* key_bytes is always 4 in this implementation.  Any out pointer may be NULL. */
pk_status pk_plan_pack_info(const pk_plan* plan, int32_t p, int32_t* dim, int32_t* dtype,
                            int64_t* total_rows, int32_t* n_fields, int32_t* n_tables,
                            int32_t* key_bytes);
/* fields_out: host, room for the pack's n_fields entries; ascending field index. */
pk_status pk_plan_pack_fields(const pk_plan* plan, int32_t p, int32_t* fields_out);
pk_status pk_plan_table_slot(const pk_plan* plan, int32_t table, int32_t* pack, int64_t* base_row);
pk_status pk_plan_field_col(const pk_plan* plan, int32_t field, int64_t* col_offset);
int64_t   pk_plan_out_dim(const pk_plan* plan);   /* sum of dims over fields; -1 if plan is NULL */

/* Upper bound of the workspace needed for a call with this B and nnz; depends
 * on no data.  Returns 0 on error (see pk_last_error). */
size_t    pk_workspace_bytes(const pk_plan* plan, int32_t B, int64_t nnz);

/* ---- forward (Sec. II-D Unique -> Gather -> SegmentReduction, packed per
 * Sec. III-B) ------------------------------------------------------------------
 * W:        host array of n_packs DEVICE pointers; W[p] is pack p's stacked
 *           table [total_rows, dim], row-major, fp32 or bf16 per the pack dtype.
 * ids:      device, int64 [nnz]; bags are field-major: bag g = f*B + b owns
 *           ids[offsets[g] .. offsets[g+1]).  Any 64-bit value is a valid ID:
 *           it is read as unsigned and folded modulo the table's rows.
 * offsets:  device, int32 [n_fields*B + 1], non-decreasing, offsets[0] = 0,
 *           offsets[n_fields*B] = nnz.
 * out:      device, fp32 [B, out_row_stride], out_row_stride >= out_dim;
 *           columns [0, out_dim) of every row are overwritten.
 * workspace: device, 256-byte aligned, >= pk_workspace_bytes(plan, B, nnz).
 *           It carries the dedup context (keys, unique, inverse, segment lists)
 *           from pk_forward to the pk_backward_update that follows.
 * hip_stream: hipStream_t (NULL = default stream).
 * Offsets that violate the contract (offsets[0] != 0, offsets[n_fields*B] != nnz,
 * a bag that ends before it begins or reaches outside its field's range) raise
 * bit 0 of the error word of the packs they touch (of every pack, when it is the
 * first or last offset of a field that is wrong); see pk_ctx_error.  Such a pack's
 * results are undefined, but no read or write leaves the caller's buffers and
 * all kernels still terminate.
 * Small batches (nnz < 2^19) run as ONE launch whose blocks sum each other's
 * counts through descriptors in device memory that the library owns and that
 * are shared by all calls on a plan: such calls on one plan must follow one
 * another (one stream, or streams ordered by events as for the two stages
 * below).  A block's wait for another block is bounded; giving up raises bit 1
 * of the error word. */
pk_status pk_forward(const pk_plan* plan, void* const* W,
                     const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz,
                     float* out, int64_t out_row_stride,
                     void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- the forward pass for callers that cannot allocate -------------------------
 * For callers that may not allocate device memory around the call: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * kernels as pk_forward, with the workspace, the plan's device metadata and the
 * scan descriptors in a static device array of 32 MiB that the library holds on
 * every GPU it runs on until the process ends; neither this call nor anything it
 * runs calls hipMalloc, hipFree or another allocating routine (no internal streams
 * or events either: every kernel runs on hip_stream).  Arguments as for pk_forward,
 * without the workspace.  PK_EWORKSPACE when the plan's metadata plus
 * pk_workspace_bytes(plan, B, nnz) exceed the 32 MiB.  All calls on one GPU share
 * that array: calls that overlap on one GPU race, and the dedup context of a call
 * (there is no pointer to hand to pk_backward_update) lasts until the next call. */
pk_status pk_forward_static(const pk_plan* plan, void* const* W,
                            const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz,
                            float* out, int64_t out_row_stride, void* hip_stream);

/* ---- backward + update (Sec. II-D: mirror of the forward pass; Adagrad from
 * the workload configurations) -------------------------------------------------
 * For every distinct key u of the preceding pk_forward (same plan, B, nnz and
 * workspace):
 *   g = sum over its occurrences of grad_out[b, col(f) .. col(f)+dim) * (1/L for mean)
 *   A[row] += g*g ;  W[row] -= lr * g / (sqrt(A[row]) + eps)
 * Rows of keys that do not occur are neither read nor written.  For a pack whose
 * error word that pk_forward raised (pk_ctx_error), nothing is read or written:
 * its W and A stay as they are.
 * A:        host array of n_packs DEVICE pointers, fp32 [total_rows, dim].
 * grad_out: device, fp32 [B, grad_row_stride]. */
pk_status pk_backward_update(const pk_plan* plan, void* const* W, float* const* A,
                             const float* grad_out, int64_t grad_row_stride,
                             int32_t B, int64_t nnz,
                             float lr, float eps,
                             void* workspace, size_t ws_bytes, void* hip_stream);

/* ---- D-Interleaving (Sec. III-C, Eq. 2): the layer on micro-batches -------------
 * A batch is cut into micro-batches that pass through the layer one after the
 * other, each with a workspace of its own size, so that the memory that grows
 * with the batch is bounded; stages of different micro-batches that use
 * different resources run side by side.  The forward pass is offered in its two
 * stages for that: the dedup of a micro-batch (H1 + H2: integer work that reads
 * no table) may run on another stream while the previous micro-batch is pooled
 * and updated.
 *
 * pk_forward_dedup + pk_forward_pool on the same workspace, B and nnz, in this order, compute
 * exactly what pk_forward computes (pk_forward may share launches between the
 * two stages).  Arguments as for pk_forward.  The caller orders the streams:
 * pk_forward_pool after the pk_forward_dedup of its workspace, pk_backward_update after the
 * pool stage, and a pool stage that must see an update after that update. */
pk_status pk_forward_dedup(const pk_plan* plan, const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz,
                   void* workspace, size_t ws_bytes, void* hip_stream);
pk_status pk_forward_pool(const pk_plan* plan, void* const* W, int32_t B, int64_t nnz,
                  float* out, int64_t out_row_stride,
                  void* workspace, size_t ws_bytes, void* hip_stream);

/* Eq. 2: BS_micro = min over the layer's operators of RBound_op / RInstance_op,
 * for the two resources of this layer that grow with the batch:
 *   - the workspace: RInstance from pk_workspace_bytes at the observed
 *     occurrences per sample (nnz / B of a warm-up batch; the part of the
 *     workspace that does not depend on the batch is taken off the bound first),
 *     RBound = ws_bound_bytes;
 *   - the activations: 8 * out_dim bytes per sample (pooled output and its
 *     gradient, fp32), RBound = act_bound_bytes.
 * A bound of 0 means "no bound".  The result is evened out as the paper does
 * (micro-batches of equal size): with M = ceil(B / BS_micro) micro-batches it is
 * ceil(B / M).  Returns 0 if not even one sample fits, -1 on bad arguments.
 * Host only. */
int32_t pk_micro_batch_size(const pk_plan* plan, int32_t B, int64_t nnz,
                            size_t ws_bound_bytes, size_t act_bound_bytes);

/* ---- HybridHash (Sec. III-D, Alg. 1): a Hot-storage in front of the tables -----
 * The pack's table passed as W_cold / A_cold is the Cold-storage and holds every
 * row; it only has to be device-ACCESSIBLE, so it may be pinned host memory
 * (hipHostMalloc) read and written by the kernels over the bus.  The Hot-storage
 * is a small device array holding, and taking the updates of, the rows queried
 * most often.  FCounter counts, per row, the iterations in which the row was
 * queried (the layer queries the distinct rows of a batch: Gather follows Unique).
 * One iteration = pk_hh_forward, pk_hh_backward_update, pk_hh_end_iteration:
 *   itr <  warmup_iters: every row is served by the Cold-storage, FCounter counts;
 *   itr >= warmup_iters: a row found in the Hot-storage is read and updated there,
 *     the others in the Cold-storage; FCounter counts; when itr is a multiple of
 *     flush_iters the Hot-storage is refreshed to hold the top-k rows of
 *     FCounter (larger count first, equal counts by smaller row; counts are
 *     compared up to 65535: rows queried in that many iterations or more are
 *     equally hot; rows never queried do not enter; k = hot_rows): rows that leave are written back to
 *     the Cold-storage, rows that enter are loaded, rows that stay keep their slot.
 * The Hot-storage never changes a value the layer computes.  All buffers belong
 * to the caller; pk_hh_init must run once before the first iteration. */
typedef struct {
    void*     W_cold;    /* device-accessible, [total_rows, dim], the pack's dtype        */
    float*    A_cold;    /* device-accessible, fp32 [total_rows, dim]                     */
    void*     W_hot;     /* device, [hot_rows, dim], the pack's dtype                     */
    float*    A_hot;     /* device, fp32 [hot_rows, dim]                                  */
    int32_t*  slot_of;   /* device, [total_rows]: the row's slot in the Hot-storage or -1 */
    uint32_t* hot_row;   /* device, [hot_rows]: the row each used slot holds (any order)  */
    uint32_t* fcounter;  /* device, [total_rows]                                          */
    int64_t   hot_rows;  /* k, the capacity of the Hot-storage in rows (>= 0)             */
} pk_hh_pack;

/* Device scratch needed by pk_hh_end_iteration (256-byte aligned) for these packs
 * (their hot_rows matter); 0 on error.  packs: host array of n_packs entries. */
size_t    pk_hh_scratch_bytes(const pk_plan* plan, const pk_hh_pack* packs);
/* packs: host array of n_packs entries.  Empties the Hot-storage bookkeeping
 * (slot_of = -1, FCounter = 0).  Enqueues on hip_stream. */
pk_status pk_hh_init(pk_plan* plan, const pk_hh_pack* packs, void* hip_stream);
/* As pk_forward / pk_backward_update, with rows read and updated where they live. */
pk_status pk_hh_forward(const pk_plan* plan, const pk_hh_pack* packs,
                        const int64_t* ids, const int32_t* offsets, int32_t B, int64_t nnz,
                        float* out, int64_t out_row_stride,
                        void* workspace, size_t ws_bytes, void* hip_stream);
pk_status pk_hh_backward_update(const pk_plan* plan, const pk_hh_pack* packs,
                                const float* grad_out, int64_t grad_row_stride, int32_t B, int64_t nnz,
                                float lr, float eps, void* workspace, size_t ws_bytes, void* hip_stream);
/* The bookkeeping of Alg. 1 for the batch of the preceding pk_hh_forward (same B,
 * nnz, workspace): FCounter, and the reload when it is due.  queried / hits: host
 * arrays of n_packs entries or NULL: distinct rows queried by the batch and how
 * many of them were in the Hot-storage; *flushed (or NULL): whether a reload took
 * place.  SYNCHRONISES hip_stream when it returns counts or reloads. */
pk_status pk_hh_end_iteration(pk_plan* plan, const pk_hh_pack* packs, int64_t itr,
                              int32_t warmup_iters, int32_t flush_iters, int32_t B, int64_t nnz,
                              const void* workspace, size_t ws_bytes, void* scratch, size_t scratch_bytes,
                              void* hip_stream, int64_t* queried, int64_t* hits, int32_t* flushed);
/* Rows currently in pack p's Hot-storage (host-side count). */
pk_status pk_hh_hot_count(const pk_plan* plan, int32_t p, int64_t* n_hot);

/* ---- Partition (Sec. II-D operator list; Sec. III-B: fused with Unique), one GPU's share ---------
 * On several workers the rows of a packed table are dealt to the workers, the distinct keys of a batch are
 * split by the worker that holds their rows, and only the keys and rows of other workers travel (Shuffle).
 * This call is the split as one GPU sees it, for pack p of the preceding pk_forward (same plan, B, nnz,
 * workspace): row r belongs to worker r mod n_owners (the paper does not say how rows are dealt), and
 *   part_keys    device, uint32 [>= distinct keys of the pack; nnz always does]: the pack's distinct keys
 *                regrouped by owner, owner 0 first, ascending inside an owner
 *   part_index   device, int32, same length: where each of them stands in the pack's `unique` list
 *                (where Stitch puts the row that comes back for it)
 *   part_offsets device, int32 [n_owners + 1]: start of every owner's group; the last entry is the number
 *                of distinct keys
 * scratch: device, >= pk_partition_scratch_bytes(plan, nnz, n_owners).  1 <= n_owners <= 64.
 * Enqueues on hip_stream. */
size_t    pk_partition_scratch_bytes(const pk_plan* plan, int64_t nnz, int32_t n_owners);
pk_status pk_partition_unique(const pk_plan* plan, const void* workspace, size_t ws_bytes, int32_t B, int64_t nnz,
                              int32_t p, int32_t n_owners, uint32_t* part_keys, int32_t* part_index,
                              int32_t* part_offsets, void* scratch, size_t scratch_bytes, void* hip_stream);

/* ---- parity access to the context saved in the workspace ---------------------
 * SYNCHRONISES the device (copies a few bytes of the header back).  Returns
 * device pointers into the workspace, valid until the next pk_forward:
 *   keys            uint32 [nnz_p]      packed key per occurrence, in packed order
 *   unique          uint32 [n_unique]   distinct keys, ascending
 *   inverse         int32  [nnz_p]      index of each occurrence's key in unique
 *   packed_offsets  int32  [k_p*B + 1]  bag boundaries in the packed order
 *   seg_offsets     int32  [n_unique+1] occurrences with a smaller key, per distinct key
 * and the host values nnz_p and n_unique.  Any out pointer may be NULL. */
pk_status pk_ctx_pack(const pk_plan* plan, const void* workspace, int32_t B, int64_t nnz, int32_t p,
                      const uint32_t** keys, const uint32_t** unique, const int32_t** inverse,
                      const int32_t** packed_offsets, const int32_t** seg_offsets,
                      int64_t* nnz_p, int64_t* n_unique);
/* Device error word of the last pk_forward on this workspace: the OR over the
 * packs' words (0 = inputs passed the checks).  SYNCHRONISES.  bit 0: offsets
 * rejected (see pk_forward); bit 1: a block waited too long for another block's
 * counts.  A pack whose word is set is skipped by pk_backward_update: its
 * tables and accumulators stay as they are. */
pk_status pk_ctx_error(const pk_plan* plan, const void* workspace, int32_t* error_word);

/* ---- per-kernel timing (for the benchmark's roofline figures) -----------------
 * With profiling on, every kernel launch is bracketed by HIP events on the
 * launch stream.  pk_profile_read synchronises, adds up the elapsed time per
 * kernel name since the last read, and fills up to max_entries entries (names
 * are static strings owned by the library).  Returns the number of entries. */
pk_status pk_profile_enable(pk_plan* plan, int32_t enable);
int32_t   pk_profile_read(pk_plan* plan, const char** names, double* total_ms, int64_t* launches,
                          int32_t max_entries);

const char* pk_last_error(void);   /* host, thread-local, never NULL */

#ifdef __cplusplus
}
#endif
#endif /* PK_H */
