/*
 * ffsnap.h -- C ABI of the MI355X snapshot library (libffsnap.so).
 *
 * The library implements the data-moving step of FFTrainer's state management on one GPU:
 *   - "fast snapshot" (section 4.2): every iteration the worker's unique training state, a list
 *     of tensors, is copied without serialisation into one pre-allocated contiguous buffer,
 *     whose size is known up front (12 bytes per parameter for Adam: fp32 master, m, v);
 *   - state loading on failover (section 3.1 steps 5-6, section 3.3): a newcomer receives that
 *     buffer and loads its tensors from it;
 *   - snapshot right after the optimizer update (section 6.2).
 * The paper copies device-to-host into an RDMA buffer and assumes fail-stop; this library keeps
 * the buffer on the device, cuts it into fixed-size chunks "ready to send", and adds a CRC32C
 * per chunk so the receiver can verify what it got.
 *
 * Definitions (N = total payload bytes, C = chunk_bytes):
 *   stream   T = seg_0 || seg_1 || ...        raw little-endian bytes, order of segs[], no padding
 *   buffer     = T || zeros up to n_chunks*C  n_chunks = ceil(N / C)
 *   crcs[j]    = CRC32C(buffer[jC, (j+1)C))   Castagnoli polynomial 0x1EDC6F41, reflected,
 *                                             init and final XOR 0xFFFFFFFF; zero tail included
 *
 * Conventions for every call:
 *   - Pointers marked DEVICE address GPU memory that the caller allocates, owns and keeps alive
 *     until the stream work has completed; pointers marked HOST are ordinary host memory that
 *     is only read during the call.  The library owns nothing but the plan.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it and the call returns without synchronising; results stay on the device.
 *   - Return value: FF_OK (0) or a negative ff_status.  Nothing throws, nothing aborts.
 *     Corruption found by ff_restore is reported through bad[] / n_bad, never as an error code.
 *   - A plan is immutable after ff_snapshot_plan has returned: no call writes to it or to its
 *     device tables.  Calls on one plan may run concurrently, from several host threads and on
 *     several streams, as long as their output arrays (chunks, crcs, bad, n_bad, and for restore
 *     and the optimizer steps the plan's tensors) differ.  Intermediate results live in the
 *     output arrays themselves: while a call is in flight crcs[] / bad[] hold partial sums.
 *   - Segments must not overlap each other, the chunk buffer or the crc arrays.
 *   - ff_pack, ff_restore, ff_restore_chunks and the optimizer steps allocate nothing, copy nothing
 *     and only launch kernels; host arrays they are given (gradient pointers, chunk ids) are read
 *     during the call and travel to the device inside kernel arguments.  They can therefore be
 *     recorded into a HIP graph, which then replays with the pointers it was captured with.
 *   - A plan belongs to the device that was current when it was built; device calls made with
 *     another device current return FF_ERR_INVALID.
 */
#ifndef FFSNAP_H
#define FFSNAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ff_plan ff_plan; /* opaque */

typedef enum {
    FF_OK = 0,
    FF_ERR_NULL = -1,    /* a required pointer is NULL                                          */
    FF_ERR_INVALID = -2, /* bad chunk size, misaligned pointer, nbytes not a multiple of the
                            element size, unknown dtype/kind/flag, incomplete parameter group   */
    FF_ERR_EMPTY = -3,   /* the segments hold no bytes at all                                   */
    FF_ERR_NOMEM = -4,   /* host or device allocation failed                                    */
    FF_ERR_HIP = -5,     /* a HIP runtime call or a kernel launch failed                        */
    FF_ERR_HOST_ONLY = -6, /* device work asked of a plan built with FF_PLAN_HOST_ONLY          */
    FF_ERR_TOO_LARGE = -7, /* input beyond the fixed capacity of an entry point that allocates
                              nothing                                                           */
    FF_ERR_LAYOUT = -8     /* the buffer was packed for another layout (ff_restore_checked)     */
} ff_status;

typedef enum { FF_BF16 = 1, FF_F32 = 2, FF_F16 = 3 } ff_dtype;

/* Role of a segment in the fused optimizer step; RAW segments are only ever copied. */
typedef enum {
    FF_KIND_RAW = 0,
    FF_KIND_W16 = 1,    /* 16-bit working weights: bf16, or fp16 (one format per plan) */
    FF_KIND_MASTER = 2, /* fp32 master weights             */
    FF_KIND_M = 3,      /* fp32 Adam first moment          */
    FF_KIND_V = 4       /* fp32 Adam second moment         */
} ff_kind;

typedef struct {
    void *ptr;         /* DEVICE; aligned to the element size (2 or 4), not necessarily to 16   */
    uint64_t nbytes;   /* multiple of the element size; 0 is allowed (the segment is skipped)   */
    uint32_t dtype;    /* ff_dtype                                                              */
    uint32_t kind;     /* ff_kind                                                               */
    uint32_t param_id; /* groups the W16/MASTER/M/V segments of one parameter; ignored for RAW  */
    uint32_t reserved; /* must be 0                                                             */
} ff_segment;

/* ff_snapshot_plan flags */
#define FF_PLAN_HOST_ONLY 1u /* build the layout only: no device memory is touched, queries work,
                                device calls return FF_ERR_HOST_ONLY (lets a sender or a test
                                compute sizes and the layout id without a GPU)                  */
/* Tuning fields of the plan flags; 0 selects the defaults, results never depend on them.
 *   bits 8..15   log2 of the tile size in bytes (the stream range one wavefront folds; clamped to
 *                [10, log2(chunk_bytes)]; default 15)
 *   bits 16..18  bit 18 set: bits 16..17 choose non-temporal accesses on the tensor side (bit 16)
 *                and on the chunk-buffer side (bit 17); default both
 *   bits 19..23  order in which workgroups take tiles: 0 = default, n in 1..29 = every XCD takes
 *                runs of 2^(n-1) consecutive workgroup tiles, 31 = plain launch order (30 is
 *                FF_ERR_INVALID: a round over the 8 XCDs would exceed the 32-bit launch index)    */
#define FF_PLAN_TILE_LOG2(n) (((uint32_t)(n) & 0xFFu) << 8)
#define FF_PLAN_CACHE_HINT(h) (0x40000u | (((uint32_t)(h) & 3u) << 16))
#define FF_PLAN_XCD_ORDER(n) (((uint32_t)(n) & 31u) << 19)

/* ff_restore flags */
#define FF_RESTORE_VERIFY_ONLY 1u /* recompute and compare CRCs, write bad[]/n_bad, scatter nothing */
#define FF_RESTORE_SKIP_BAD 2u    /* verify first, then scatter only the chunks whose CRC matched:
                                     tensor ranges covered by a bad chunk keep their old contents
                                     (the buffer is read twice: 3 B of traffic per payload byte)  */

#define FF_MIN_CHUNK_BYTES 1024ull
#define FF_MAX_CHUNK_BYTES (1ull << 30)

/*
 * Lay out a snapshot (section 4.2: the engine walks the training configuration once and
 * computes the buffer size).  segs: HOST array of n_segs descriptors, copied.  chunk_bytes: a
 * power of two in [FF_MIN_CHUNK_BYTES, FF_MAX_CHUNK_BYTES].  The plan keeps small device
 * tables (segment pointers and offsets, a tile-to-segment index, CRC constants, the work list of
 * the optimizer steps) on the device that is current at the time of the call.
 * Errors: NULL -> FF_ERR_NULL; bad chunk size / alignment / dtype / kind / reserved / flags ->
 * FF_ERR_INVALID; N == 0 -> FF_ERR_EMPTY; allocation -> FF_ERR_NOMEM; HIP -> FF_ERR_HIP.
 * On error *out is set to NULL.
 */
int ff_snapshot_plan(const ff_segment *segs, uint64_t n_segs, uint64_t chunk_bytes, uint32_t flags,
                     ff_plan **out);

/* Frees the plan and its device tables.  NULL is ignored.  The caller must have synchronised
 * every stream that still uses the plan. */
void ff_plan_destroy(ff_plan *plan);

uint64_t ff_plan_payload_bytes(const ff_plan *plan); /* N                                   */
uint64_t ff_plan_num_chunks(const ff_plan *plan);    /* ceil(N / chunk_bytes)               */
uint64_t ff_plan_buffer_bytes(const ff_plan *plan);  /* num_chunks * chunk_bytes            */
uint64_t ff_plan_chunk_bytes(const ff_plan *plan);
uint64_t ff_plan_num_segments(const ff_plan *plan);  /* non-empty segments                  */
uint64_t ff_plan_num_params(const ff_plan *plan);    /* complete W16/MASTER/M/V groups      */
/* CRC32C over the little-endian uint64 sequence (chunk_bytes, nbytes of every non-empty segment
 * in order): equal ids on sender and receiver mean the two layouts agree. */
uint32_t ff_plan_layout_id(const ff_plan *plan);
/* Stream range [*begin, *end) of non-empty segment i; FF_ERR_INVALID if i is out of range. */
int ff_plan_segment_range(const ff_plan *plan, uint64_t i, uint64_t *begin, uint64_t *end);

/*
 * Checkpoint razor (section 4.2): which of a worker's segments are unique state, to be
 * snapshotted every iteration, and which are redundant across the data-parallel group, to be
 * saved only at recovery time by one healthy worker ("lazy backup").  The two rules:
 *   (1) data-parallel degree > 1                                  -> model weights are redundant;
 *   (2) data-parallel degree > 1 and no distributed optimizer     -> optimizer states are redundant.
 * FF_KIND_W16 segments are the model weights, FF_KIND_MASTER / M / V the optimizer states (the
 * 12 bytes per parameter of the paper's size law); FF_KIND_RAW segments have no known role and
 * always count as unique.  Host-only; no GPU is touched.
 */
typedef struct {
    uint32_t dp_degree;             /* d >= 1 */
    uint32_t distributed_optimizer; /* 0 / 1: optimizer states sharded over the DP group */
} ff_razor_config;

#define FF_RAZOR_UNIQUE 0u    /* the per-iteration snapshot list */
#define FF_RAZOR_REDUNDANT 1u /* the lazy-backup list (the complement) */

/*
 * Writes to out_indices (HOST, room for n_segs entries) the indices, ascending, of the segments
 * of segs[] (HOST) that fall into `which`, and their number to *n_out.  A plan for the selection
 * is then built from those segments in that order.  FF_ERR_NULL / FF_ERR_INVALID (dp_degree 0,
 * unknown `which`, kind or flag value) as usual.
 */
int ff_razor_select(const ff_segment *segs, uint64_t n_segs, const ff_razor_config *cfg,
                    uint32_t which, uint64_t *out_indices, uint64_t *n_out);

/*
 * Snapshot (section 4.2, "fast snapshot"): gather the segments into `chunks` and write one
 * CRC32C per chunk.  chunks: DEVICE, 16-byte aligned, ff_plan_buffer_bytes() bytes, every byte
 * of it is written (the tail of the last chunk with zeros).  crcs: DEVICE, num_chunks uint32.
 */
int ff_pack(const ff_plan *plan, void *chunks, uint32_t *crcs, void *hip_stream);

/*
 * Snapshot into host memory (section 4.2: the snapshot is copied device-to-host into a
 * pre-allocated buffer, from where it is streamed to the next worker).  The snapshot is packed
 * in slices of slice_chunks chunks on pack_stream; as soon as a slice and its CRCs are complete
 * they are copied to host_chunks / host_crcs on copy_stream, while the next slice is being
 * packed.  chunks / crcs: DEVICE staging of the full snapshot, as for ff_pack (it also holds the
 * snapshot afterwards).  host_chunks (buffer_bytes) and host_crcs (num_chunks uint32): HOST,
 * ideally pinned (hipHostMalloc); pageable memory works but the copies then do not overlap.
 * The two streams should differ (both default priority); the call returns without
 * synchronising: the host buffers are complete once copy_stream has been synchronised.  Keeping
 * the two most recent snapshots (section 4.2) is the caller alternating two host buffers.
 */
int ff_pack_to_host(const ff_plan *plan, void *chunks, uint32_t *crcs, void *host_chunks,
                    uint32_t *host_crcs, uint64_t slice_chunks, void *pack_stream,
                    void *copy_stream);

/*
 * State loading on failover (section 3.1 steps 5-6, section 3.3): recompute the CRC32C of every
 * chunk of `chunks`, set bad[j] = (recomputed != crcs[j]) and *n_bad = sum(bad), and copy every
 * segment's bytes out of the buffer into the plan's tensors -- from good and bad chunks alike:
 * the caller must treat tensor ranges that a bad chunk covers as invalid.  chunks: DEVICE,
 * 16-byte aligned, buffer_bytes.  crcs: DEVICE, num_chunks.  bad: DEVICE, num_chunks uint32,
 * each set to 0 or 1.  n_bad: DEVICE, one uint64.  flags: 0, FF_RESTORE_VERIFY_ONLY or
 * FF_RESTORE_SKIP_BAD.
 */
int ff_restore(const ff_plan *plan, const void *chunks, const uint32_t *crcs, uint32_t *bad,
               uint64_t *n_bad, uint32_t flags, void *hip_stream);

/*
 * ff_restore for a buffer that arrives from another worker (section 3.1 steps 5-6: the state
 * controller forwards a healthy worker's state to the newcomer): sender_layout_id is the sender's
 * ff_plan_layout_id(), shipped along with the buffer.  If it differs from this plan's id the two
 * workers disagree on chunk size or tensor sizes and the buffer's bytes would land in the wrong
 * tensors: FF_ERR_LAYOUT is returned, nothing is enqueued, no tensor, bad[] or n_bad is written.
 * Otherwise exactly ff_restore.
 */
int ff_restore_checked(const ff_plan *plan, uint32_t sender_layout_id, const void *chunks,
                       const uint32_t *crcs, uint32_t *bad, uint64_t *n_bad, uint32_t flags,
                       void *hip_stream);

/*
 * Selective state loading: the same as ff_restore for the n_ids chunks named in chunk_ids only
 * (HOST array, strictly ascending, each < num_chunks) -- the chunks a worker re-fetched after a
 * first restore flagged them, or the part of the state another source supplies (section 4.2:
 * state that instant checkpointing cannot supply comes from a fallback).  bad[j] is written for
 * the listed chunks alone, *n_bad counts the bad ones among them, tensor bytes outside the
 * listed chunks are not touched.  Flags as for ff_restore.  FF_ERR_INVALID for an id out of
 * range or a list that is not strictly ascending.  n_ids == 0 only sets *n_bad = 0.
 */
int ff_restore_chunks(const ff_plan *plan, const void *chunks, const uint32_t *crcs,
                      const uint64_t *chunk_ids, uint64_t n_ids, uint32_t *bad, uint64_t *n_bad,
                      uint32_t flags, void *hip_stream);

/* Which tensor ranges a chunk covers: [*begin, *end) is the chunk's payload range in stream
 * coordinates (clipped to N), and the non-empty segments *first_seg .. *first_seg + *n_seg - 1
 * intersect it (use ff_plan_segment_range for their stream ranges).  Host-only query. */
int ff_plan_chunk_span(const ff_plan *plan, uint64_t chunk, uint64_t *first_seg, uint64_t *n_seg,
                       uint64_t *begin, uint64_t *end);

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    uint32_t step; /* t >= 1 of the bias corrections */
} ff_adam_hparams;

/*
 * Optimizer update with the snapshot taken in the same pass (section 6.2: the optimizer state
 * is checkpointed immediately after each update).  For every parameter group of the plan one
 * decoupled-weight-decay Adam step in fp32, each operation rounded separately, in this order:
 *     g = float(grad);  p = master*decay;  m' = b1*m + omb1*g;  v' = b2*v + (omb2*g)*g;
 *     d = sqrt(v')/bc2s + eps;  p' = p - step_size*(m'/d);  w' = bf16_rne(p')
 * with decay = 1 - lr*wd, omb1 = 1 - b1, omb2 = 1 - b2, step_size = lr/(1 - b1^t),
 * bc2s = sqrt(1 - b2^t) evaluated in double and rounded once to fp32.  master, m, v and the bf16
 * weights are overwritten in place and the same bytes are written at their stream offsets in
 * `chunks`; RAW segments are copied unchanged; crcs as in ff_pack.  The result equals ff_pack
 * run after an unfused update.  A new master, m or v that is NaN is stored as the canonical quiet
 * NaN 0x7FC00000 (IEEE 754 leaves sign and payload of a produced NaN open and processors differ;
 * the snapshot and its CRCs must not), and w' is rounded from the stored value: 0x7FC0.  grads: HOST array of ff_plan_num_params() DEVICE pointers to
 * bf16 gradients (2-byte aligned), indexed by param_id rank (ascending param_id); read only.
 * FF_ERR_INVALID if the plan has an incomplete group, mismatched element counts, or step == 0.
 */
int ff_adam_step_snapshot(const ff_plan *plan, const void *const *grads, const ff_adam_hparams *hp,
                          void *chunks, uint32_t *crcs, void *hip_stream);

/*
 * The same step for fp16 training with a loss scale (section 7.1: the evaluated models train in
 * fp16).  The plan's working weights are FF_F16; grads point to fp16 gradients of a loss that
 * was multiplied by S, and inv_loss_scale = 1/S:
 *     g = float(grad) * inv_loss_scale   (one rounded fp32 multiplication)
 * then the arithmetic of ff_adam_step_snapshot, and w' = fp16_rne(p') (overflow gives infinity;
 * the canonical NaN that a NaN result is stored as becomes 0x7E00).  n_nonfinite: DEVICE, one uint64,
 * 8-byte aligned, or NULL: receives the number of gradient elements that are infinite or NaN.
 * The update is applied to every element regardless; a caller that lowers S on overflow goes
 * back to the previous snapshot (the paper keeps the two most recent ones, section 4.2).
 * FF_ERR_INVALID also if the plan's working weights are bf16 (and ff_adam_step_snapshot
 * returns it for an fp16 plan).
 */
int ff_adam_step_snapshot_f16(const ff_plan *plan, const void *const *grads,
                              const ff_adam_hparams *hp, float inv_loss_scale,
                              uint64_t *n_nonfinite, void *chunks, uint32_t *crcs,
                              void *hip_stream);

/*
 * The same step with the optimizer state kept in the snapshots themselves.  The paper holds the
 * two most recent snapshots and alternates between them (section 4.2) and snapshots right after
 * every update (section 6.2); here the update of step t reads the old master, m and v of every
 * parameter group from `prev_chunks`, the snapshot of step t-1, at the segments' stream offsets,
 * and writes the new master, m, v and 16-bit weights into `chunks`.  The plan's MASTER, M and V
 * tensors are neither read nor written (they may be views into the snapshot buffers, or unused);
 * the W16 tensors receive the new working weights as in the other two steps; gradients and RAW
 * segments are read from their tensors.  Arithmetic, rounding, crcs and the zero tail are those
 * of ff_adam_step_snapshot (bf16 plan: inv_loss_scale must be 1 and n_nonfinite NULL) or of
 * ff_adam_step_snapshot_f16 (fp16 plan), so the result equals that step run on tensors holding
 * the state of `prev_chunks`.  The CRCs of `prev_chunks` are not checked here (ff_restore with
 * FF_RESTORE_VERIFY_ONLY does that).  Per element it moves 14 bytes in and 16 out, where the
 * in-place steps move 14 in and 28 out.
 * prev_chunks: DEVICE, 16-byte aligned, ff_plan_buffer_bytes() long, read only; it must not
 * overlap `chunks` (FF_ERR_INVALID).
 */
int ff_adam_step_chained(const ff_plan *plan, const void *const *grads, const ff_adam_hparams *hp,
                         float inv_loss_scale, uint64_t *n_nonfinite, const void *prev_chunks,
                         void *chunks, uint32_t *crcs, void *hip_stream);

/* Test helper: CRC32C of nbytes at dev_buf (DEVICE, 16-byte aligned) into *dev_out (DEVICE),
 * computed by the same tile and combine kernels as ff_pack.  Allocates and frees a small
 * scratch array, so it synchronises the stream before returning. */
int ff_crc32c(const void *dev_buf, uint64_t nbytes, uint32_t *dev_out, void *hip_stream);

/*
 * ff_crc32c for callers that cannot allocate or must not be synchronised: code that is being
 * captured into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and result as ff_crc32c, but the scratch memory (reduction tables and one CRC
 * register per 1 MiB of input) is a fixed array in the library's device image instead of an
 * allocation, and the call only enqueues kernels on hip_stream and returns: *dev_out is valid
 * once the stream has reached that point.  It never calls hipMalloc or hipFree.
 * Limits: nbytes <= FF_CRC32C_NOALLOC_MAX_BYTES, else FF_ERR_TOO_LARGE and nothing is enqueued.
 * The array (about 260 KiB) exists once per GPU and is shared by every call on that GPU: two
 * calls whose kernels may overlap in time (different streams) race on it and give wrong results;
 * calls on one stream are safe back to back.  The first call on a device looks up the array's
 * address and copies the tables into it with a blocking hipMemcpy, so make one eager call per
 * device before capturing it into a graph.
 */
#define FF_CRC32C_NOALLOC_MAX_BYTES (1ull << 36) /* 64 GiB */
int ff_crc32c_noalloc(const void *dev_buf, uint64_t nbytes, uint32_t *dev_out, void *hip_stream);

/* Bench helper: plain device copy of nbytes (both DEVICE, 16-byte aligned, nbytes a multiple of
 * 16, the ranges disjoint) in the access pattern of ff_pack but without the CRC: the measured
 * bandwidth ceiling printed beside the real kernels. */
int ff_copy_ceiling(void *dst, const void *src, uint64_t nbytes, void *hip_stream);

/* Bench helper: the memory traffic of the optimizer steps with nothing else -- for every
 * parameter group of the plan the same tiles, loads and stores as ff_adam_step_snapshot
 * (prev_chunks NULL: 14 bytes read, 28 written per element) or as ff_adam_step_chained
 * (prev_chunks set: 14 read, 16 written), but no arithmetic and no CRC: the new 16-bit weights are
 * the gradient's bits, master, m and v keep their values.  crcs, RAW segments and the zero tail
 * of `chunks` are not written.  The measured ceiling of this mix of streams, printed beside the
 * real steps.  Arguments as for those steps. */
int ff_mix_ceiling(const ff_plan *plan, const void *const *grads, const void *prev_chunks,
                   void *chunks, void *hip_stream);

/* Static string for a status code; for FF_ERR_HIP the text of the last HIP error seen by the
 * calling thread is appended. */
const char *ff_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* FFSNAP_H */
