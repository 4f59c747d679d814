/*
 * reft.h - C ABI of libreft: the device-side hot path of in-memory checkpointing for one rank.
 *
 * What the library does, in the paper's terms (REFT, arXiv 2310.12670):
 *   - snapshot: the rank's state tensors (parameters and optimizer states, section 1) are taken
 *     as one flat vector, the "vectorized W" that SplitParameter of Algorithm 1 cuts by index;
 *     consecutive byte ranges of it ("buckets") are gathered on the GPU and copied to a pinned
 *     host buffer asynchronously to training (section 4.1; section 6: pinned host buffers);
 *   - protect: the k snapshot shards of a node are encoded into one XOR parity unit on the
 *     device (section 4.2, Asynchronous Erasure Coding, Eq. 1; section 6: bitwise XOR);
 *   - load: a shard is copied back from host memory into the tensors (section 4.3, step 1) and a
 *     single lost shard is decoded from the parity and the survivors (section 4.2, Eq. 2;
 *     section 4.3, step 3).
 *
 * Vocabulary
 *   span    one tensor's raw bytes: a device pointer and a byte count (may be 0).
 *   stream  the tight concatenation of a shard's spans in list order, L bytes; no header, no
 *           padding.  All results are defined on the stream's bytes; values are never interpreted.
 *   bucket  a consecutive byte range [B_b, B_{b+1}) of the stream; a transport unit only: the
 *           host copy produced by reft_snapshot_pack equals the stream whatever the buckets are.
 *   plan    the sizes of the spans and buckets of a shard (no pointers, no data); k shards that
 *           are protected together share one plan (identical span sizes).
 *
 * General rules
 *   - Every function returns 0 (REFT_OK) or a negative REFT_E* code; it never throws or aborts.
 *     reft_last_error() gives a message for the calling thread's most recent failure.
 *   - "device" pointers are HIP device addresses on the plan's GPU; "host" pointers are host
 *     addresses.  Pointer *arrays* (span_ptrs, shards) are host arrays holding device addresses.
 *   - The caller owns all data buffers, the staging ring, the pinned host buffer and the HIP
 *     streams.  The library owns only the plan (host tables, their device copies, events).
 *   - Device and pinned memory is allocated by reft_plan_create, reft_ckpt_create and the first
 *     rotated call for a given (k, member) only.  The data-moving calls allocate none and never
 *     wait for the whole device; they block the calling thread only in one case: a call that
 *     brings a pointer array the plan has not seen lately may have to wait for the kernels that
 *     still read the cached table whose room it takes (see reft_plan_create).  (The optional
 *     transports "dma_streams" = 2 and "graph_copies" make a helper stream / a graph on the first
 *     call that uses them.)
 *   - The data-moving calls enqueue work on the given streams and return; results are complete
 *     when those streams (or reft_snapshot_wait / reft_restore_wait) have been synchronised.
 *     Source data must not be modified, and pointer arrays' targets not freed, before that.
 *     The pointer arrays themselves are copied before the call returns.
 *   - A plan is bound to the GPU that was current at reft_plan_create; calls on one plan must not
 *     be issued from two host threads at once.  Streams stay at the default priority.
 *   - reft_stream is a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef REFT_H
#define REFT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define REFT_OK               0
#define REFT_EINVAL         (-1)  /* null pointer, k out of range, T == 0, zero-length bucket     */
#define REFT_ESIZE          (-2)  /* a buffer is too small or a length does not match the plan    */
#define REFT_EHIP           (-3)  /* a HIP runtime call failed; text in reft_last_error()         */
#define REFT_EUNRECOVERABLE (-4)  /* more than one shard lost: beyond what one parity can decode  */
#define REFT_EBUSY          (-5)  /* reft_ckpt_begin while an earlier commit has not landed yet      */

#define REFT_MAX_K 32             /* most shards (or survivors + parity) in one call              */

typedef struct reft_plan reft_plan;
typedef void *reft_stream;

/* ---- S0: plan (host integer arithmetic; done once and reused for every snapshot) -------------
 * The sizing and splitting that Algorithm 1 performs on the host per stage: prefix sums of the
 * span sizes, the bucket boundaries, and the tile table the kernels walk.
 *
 * span_nbytes[T]    host array, byte size of each span in stream order (zeros allowed), T >= 1.
 * uniform_bucket    if non-zero: buckets of this many bytes (the last one shorter);
 *                   bucket_nbytes/NB are ignored.
 * bucket_nbytes[NB] otherwise: host array of positive bucket lengths whose sum must equal L
 *                   (NB may be 0 only when L == 0).  With bucket_nbytes == NULL, NB == 0 and
 *                   uniform_bucket == 0 the whole stream is one bucket.
 * out               receives the plan; destroy it with reft_plan_destroy.
 * Allocates on the current GPU everything the data-moving calls will need: the device tables, the
 * events, the burst kernels' counters, the piece lists of the staged transport for the whole
 * stream, and a cache for the callers' pointer arrays (72 rows of T pointers, pinned host mirror
 * and device copy).  A call that passes pointers the cache already holds uploads nothing; up to
 * 32 tables are kept, each remembering the streams (up to 4) that last read it, and a new table
 * takes the room of the oldest ones after waiting for exactly those readers.
 * Errors: REFT_EINVAL (null out/span_nbytes, T == 0, a zero-length bucket), REFT_ESIZE (bucket
 * lengths do not sum to L), REFT_EHIP.
 */
int reft_plan_create(const uint64_t *span_nbytes, uint64_t T,
                     const uint64_t *bucket_nbytes, uint64_t NB, uint64_t uniform_bucket,
                     reft_plan **out);
void reft_plan_destroy(reft_plan *plan);                 /* NULL is allowed                       */
uint64_t reft_plan_stream_bytes(const reft_plan *plan);  /* L                                     */
uint64_t reft_plan_num_spans(const reft_plan *plan);     /* T                                     */
uint64_t reft_plan_num_buckets(const reft_plan *plan);   /* NB                                    */
uint64_t reft_plan_max_bucket_bytes(const reft_plan *plan);
/* Smallest staging ring (bytes) that holds one bucket; n slots need n times this. */
uint64_t reft_plan_staging_slot_bytes(const reft_plan *plan);
/* Byte range [*begin, *end) of bucket b.  REFT_EINVAL if b >= NB. */
int reft_plan_bucket_range(const reft_plan *plan, uint64_t b, uint64_t *begin, uint64_t *end);
/* Stream offset at which span t starts (t == T gives L).  REFT_EINVAL if t > T. */
int reft_plan_span_offset(const reft_plan *plan, uint64_t t, uint64_t *offset);
/* The kernels' work decomposition: tiles of *tile_bytes consecutive stream bytes, *ntiles of them;
 * reft_plan_tile_first_span gives the first span owning a byte of tile t (for inspection/tests). */
int reft_plan_tile_info(const reft_plan *plan, uint64_t *tile_bytes, uint64_t *ntiles);
int reft_plan_tile_first_span(const reft_plan *plan, uint64_t t, uint64_t *span);
/* The index cut of SplitParameter (Algorithm 1): floor(n * t_bubble / t_ss) with n = L bytes,
 * clamped to [0, L]; t_ss must be > 0.  Returns the cut through *cut. */
int reft_plan_split(const reft_plan *plan, double t_bubble, double t_ss, uint64_t *cut);
/* What a staged snapshot (or restore) of the whole stream consists of under the current
 * "dma_min_bytes" / "gather_min_pieces": *gather_launches kernel launches on pack_stream (runs of
 * small pieces) and *copies hipMemcpyAsync calls on copy_stream.  With *gather_launches == 0 the
 * transport is pure DMA, pack_stream carries no work, and the caller may pass one stream for both
 * (one hardware queue less: see the note on streams under reft_snapshot_pack). */
int reft_plan_staged_work(reft_plan *plan, uint64_t *gather_launches, uint64_t *copies);

/* ---- S1 + S2 + S3: bucketed snapshot of one shard into pinned host memory -----------------------
 * Bucket by bucket, in order, the shard's stream is moved from the ragged span tensors to
 * host_dst + B_b.  Two transports, chosen per call by the staging argument:
 *   staged (staging != NULL)  the transport for snapshots taken beside training.  Every piece
 *       (bucket x span) of at least "dma_min_bytes" is copied by hipMemcpyAsync on copy_stream
 *       straight from its tensor to host_dst: no kernel runs, so kernels of the training step
 *       are not disturbed.  Smaller pieces are copied the same way when few lie together; a run
 *       of at least "gather_min_pieces" consecutive small pieces within a bucket is gathered by
 *       one kernel launch on pack_stream into a slot of the staging ring and leaves as one copy
 *       (many small tensors would otherwise mean thousands of tiny transfers).  The ring's slots
 *       form two groups used alternately; the two streams synchronise through events once per
 *       group.  pack_stream may equal copy_stream (fully in order).  The tensors are read in
 *       pack_stream's order: work queued on pack_stream before the call (say, the kernel that
 *       produced a parity buffer) completes before any byte is read, also by the copies.
 *   direct (staging == NULL)  the gather kernel itself stores into the pinned host buffer across
 *       the host link: one launch per bucket on pack_stream, capped at "link_wgs" workgroups (a
 *       few dozen saturate the link).  No staging memory, no DMA, no second pass over HBM;
 *       copy_stream is not used.  Meant for times when the GPU is otherwise idle (pipeline
 *       bubbles, recovery): kernels that keep the link's write path full slow down kernels
 *       running beside them.  host_dst must be device-accessible pinned memory (hipHostMalloc),
 *       else REFT_EINVAL.
 * Streams: the HIP runtime deals streams onto a few hardware queues (4 per process by default) as
 * they are created, whether they ever get work or not, and two streams on one queue run in turn.
 * A snapshot and a restore only overlap on the link (full duplex) if their copy streams sit on
 * different queues: give each its own stream, created early, and keep the process's stream count
 * low (when reft_plan_staged_work reports no gather launches, one stream serves as pack_stream
 * and copy_stream).  Copy engines: the runtime gives a stream's copies to the lowest-numbered copy
 * engine with nothing pending when the stream chooses, and the stream keeps it until a wait for
 * another stream's event has come true.  Two consequences, both measured: with several snapshots'
 * copies queued ahead (thousands of hipMemcpyAsync calls) the choice reaches engines that move
 * host traffic at a quarter of the rate, so wait for the previous snapshot (reft_snapshot_wait, an
 * event) before queuing the next; and a restore queued while nothing is in flight can be given
 * the engine that the snapshot stream still holds, after which the two directions take turns
 * instead of overlapping: queue one direction while the other still has copies pending.
 * After the last bucket a completion event is recorded (see reft_snapshot_wait): the snapshot is
 * complete only when every bucket has landed (section 4.4: COMPLETED when all tensors are
 * snapshotted).  Postcondition: host_dst[0..L) == stream; host_dst[L..) untouched.
 *
 * span_ptrs[T]   host array of device pointers (may be NULL where the span has 0 bytes).
 * staging        NULL, or a 256-byte-aligned device buffer of staging_bytes >=
 *                reft_plan_staging_slot_bytes(plan); up to 64 slots are used.  Scratch contents;
 *                must not be shared with another call that may be in flight.
 * host_dst       host buffer of host_cap >= L bytes, pinned.
 * Errors: REFT_EINVAL, REFT_ESIZE (host_cap < L, staging smaller than one slot), REFT_EHIP.
 */
int reft_snapshot_pack(reft_plan *plan, const void *const *span_ptrs,
                       void *staging, uint64_t staging_bytes,
                       void *host_dst, uint64_t host_cap,
                       reft_stream pack_stream, reft_stream copy_stream);
/* The same for the buckets [bucket_begin, bucket_end) only: the unit a scheduler places into a
 * pipeline bubble or beside computation (Algorithm 1 launches W_bubble, the part of the flat vector
 * before the SplitParameter cut, in bubble time and the rest in computation time).  The snapshot
 * is complete when calls covering all buckets have landed.  REFT_EINVAL if the range is not within
 * [0, NB].  reft_plan_bucket_of gives the bucket that holds a stream offset (offset == L gives NB).
 */
int reft_snapshot_pack_range(reft_plan *plan, const void *const *span_ptrs,
                             void *staging, uint64_t staging_bytes,
                             void *host_dst, uint64_t host_cap,
                             uint64_t bucket_begin, uint64_t bucket_end,
                             reft_stream pack_stream, reft_stream copy_stream);
int reft_plan_bucket_of(const reft_plan *plan, uint64_t offset, uint64_t *bucket);
/* Block until every reft_snapshot_pack[_range] issued on this plan so far has fully landed on the
 * host (a call that ends on another stream than the one before it chains its completion behind
 * that call's, on the device). */
int reft_snapshot_wait(reft_plan *plan);
/* 1 if it has landed (or none was issued), 0 if still in flight, negative on error. */
int reft_snapshot_query(reft_plan *plan);

/* ---- completed / ongoing snapshot pair (section 4.4, Snapshot Management) --------------------------
 * Host memory keeps one completed snapshot while the next one is being written; the new one
 * replaces the old only when all of it has landed, so an interrupted save never damages the copy a
 * recovery would load.  A reft_ckpt tracks two caller-owned pinned buffers of `cap` >= L bytes:
 *   reft_ckpt_begin   picks the buffer that does NOT hold the newest complete snapshot, marks it
 *                     as being overwritten and returns it (*host_dst) with a new generation number;
 *   (the caller then issues reft_snapshot_pack / _range calls into *host_dst)
 *   reft_ckpt_commit  enqueues, on the stream on which the last bucket lands (copy_stream for the
 *                     staged transport, pack_stream for the direct one), a one-thread kernel that
 *                     stores the generation into a pinned flag after everything queued before it:
 *                     the COMPLETED mark of section 4.4;
 *   reft_ckpt_latest  returns the newest buffer whose flag equals the generation begun in it
 *                     (*host_src == NULL, generation 0 if there is none yet).  Never blocks.
 *   reft_ckpt_wait    blocks until every commit queued so far has landed.
 * One snapshot at a time: reft_ckpt_begin returns REFT_EBUSY while a commit queued earlier has not
 * landed (until then its buffer is neither complete nor free, and the other buffer holds the only
 * complete copy).  A snapshot that was begun and never committed (torn) may be begun again once the
 * caller has synchronised the streams it was issued on.  reft_ckpt_destroy waits for queued commits.
 * Errors: REFT_EINVAL (null arguments, commit without begin), REFT_ESIZE (cap < L), REFT_EBUSY,
 * REFT_EHIP.  Not thread-safe.
 */
typedef struct reft_ckpt reft_ckpt;
int reft_ckpt_create(reft_plan *plan, void *host_buf0, void *host_buf1, uint64_t cap,
                     reft_ckpt **out);
void reft_ckpt_destroy(reft_ckpt *ckpt);
int reft_ckpt_begin(reft_ckpt *ckpt, void **host_dst, uint64_t *generation);
int reft_ckpt_commit(reft_ckpt *ckpt, reft_stream stream);
int reft_ckpt_latest(reft_ckpt *ckpt, const void **host_src, uint64_t *generation);
int reft_ckpt_wait(reft_ckpt *ckpt);

/* ---- S1 alone / S7 alone: the gather and scatter kernels between device buffers ------------------
 * reft_pack_device:   dst_dev[0..L) = stream of the spans           (one launch over [0, L)).
 * reft_unpack_device: the spans = slices of src_dev[0..L)           (inverse of the above).
 * dst_cap >= L and src_bytes == L are checked (REFT_ESIZE).
 */
int reft_pack_device(reft_plan *plan, const void *const *span_ptrs,
                     void *dst_dev, uint64_t dst_cap, reft_stream stream);
int reft_unpack_device(reft_plan *plan, const void *src_dev, uint64_t src_bytes,
                       void *const *span_ptrs, reft_stream stream);

/* ---- S4: XOR parity over the k shards of the node (section 4.2, Eq. 1) ---------------------------
 * parity_dev[i] = S_0[i] ^ ... ^ S_{k-1}[i] for i in [0, L), where S_s is the stream of shard s
 * read in place through its span pointers (no packed copy of the shards is needed).
 *
 * shard_span_ptrs  host array of k*T device pointers, row-major: entry s*T + t is span t of
 *                  shard s.  A shard that is already packed is expressed with a 1-span plan.
 * k                1 <= k <= REFT_MAX_K (k == 1 copies the stream).
 * parity_dev       device buffer of at least L bytes; must not overlap any span.
 * Errors: REFT_EINVAL (k out of range, null), REFT_EHIP.
 */
int reft_parity_encode(reft_plan *plan, const void *const *shard_span_ptrs, uint32_t k,
                       void *parity_dev, reft_stream stream);

/* ---- S1 + S4 in one pass: parity of the k shards and the packed stream of one of them ------------
 * parity_dev as for reft_parity_encode; packed_dev[0..L) = the stream of shard `own` (what
 * reft_pack_device gives).  One kernel reads the k shards once and writes both: (k + 2) L bytes of
 * HBM traffic instead of the (k + 3) L of an encode followed by a pack ("convert local snapshot
 * segments into parity data" while they are being gathered, section 3).  For a scheduler that
 * gathers and encodes in a bubble and lets two large copies (packed shard, parity) leave beside
 * computation, or where many small tensors would be gathered by a kernel anyway.
 * The single pass is taken where the write-burst kernel applies (see "burst"), with at most 8
 * shards, parity_dev and packed_dev aligned alike modulo 16, "unroll" 4 and "nontemporal" 1, and
 * "burst_stage_bytes" <= 36864 (two LDS images per half); otherwise the call runs the encode and
 * the pack as two launches, with the same result.
 * own < k; packed_cap >= L (REFT_ESIZE); neither buffer may overlap a span or the other.
 * Errors: REFT_EINVAL, REFT_ESIZE, REFT_EHIP.
 */
int reft_parity_encode_pack(reft_plan *plan, const void *const *shard_span_ptrs, uint32_t k,
                            uint32_t own, void *parity_dev, void *packed_dev, uint64_t packed_cap,
                            reft_stream stream);

/* ---- reft_parity_encode for callers that cannot allocate ------------------------------------------
 * For code that may not call hipMalloc while it runs: work under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, same result as reft_parity_encode; the
 * call itself allocates no device or pinned memory, frees none, uses none of the plan's caches
 * and records no event.  What reft_parity_encode keeps in buffers the plan allocated - the device
 * copy of the span pointers and the write-burst kernels' counters - lives here in a static device
 * array of the library, 258.5 KiB (256 KiB of pointers, then one counter block), which every GPU
 * the library runs on holds until the process ends.  The pointers reach it as arguments of
 * small kernels (256 per launch) on `stream`; the counters are cleared by a kernel before each
 * XOR launch.
 * Limit: k * T <= 32768 span pointers, else REFT_ESIZE.
 * All calls on one GPU share the array: a call must not overlap, on another stream or from
 * another thread, with another call of this function on the same GPU (the later one would
 * overwrite the pointer table the earlier one still reads).  Calls on one stream are ordered.
 * The plan must have been created on the current GPU (that is when the array's device address
 * is looked up).  Other errors as reft_parity_encode.
 */
int reft_parity_encode_noalloc(reft_plan *plan, const void *const *shard_span_ptrs, uint32_t k,
                               void *parity_dev, reft_stream stream);

/* ---- S6: decode the single lost shard (section 4.2, Eq. 2) ---------------------------------------
 * out_dev[i] = parity[i] ^ (XOR over the surviving shards s of shards[s][i]), i in [0, L).
 *
 * (The XOR kernel's counters live in 18 KiB of static device memory of the library.)
 *
 * shards[k]   host array of device pointers to the packed streams (L bytes each) of the node's k
 *             shards; exactly one entry is NULL: the lost shard.
 * parity      device pointer, L bytes.   out_dev: device buffer of L bytes, no overlap with inputs.
 * lost_index  if not NULL, receives the index of the NULL entry.
 * Errors: REFT_EUNRECOVERABLE if two or more entries are NULL (one parity tolerates one loss per
 * group, section 4.2); REFT_EINVAL if none is NULL, k < 1 or k > REFT_MAX_K - 1, or a null
 * parity/out with L > 0; REFT_EHIP.
 */
int reft_reconstruct(const void *const *shards, uint32_t k, const void *parity, uint64_t L,
                     void *out_dev, uint32_t *lost_index, reft_stream stream);

/* ---- S6 + S7 in one pass: decode the lost shard directly into its tensors -------------------------
 * Same result as reft_reconstruct followed by reft_unpack_device, without packed copies of the
 * survivors: the k-1 surviving shards are read in place through their span pointers, the parity
 * as a contiguous stream, and the decoded bytes go straight into out_span_ptrs (Eq. 2 applied
 * span by span; section 4.3, step 3).
 *
 * shard_span_ptrs  host array of k*T device pointers, row-major as for reft_parity_encode; row
 *                  `lost` is ignored (its entries may be NULL).
 * lost             index of the lost shard, < k;  1 <= k <= REFT_MAX_K - 1.
 * parity_dev       device pointer to the L parity bytes.
 * out_span_ptrs    host array of T device pointers: the tensors that receive the lost shard.
 * Errors: REFT_EINVAL (k or lost out of range, null pointers), REFT_EHIP.
 */
int reft_reconstruct_spans(reft_plan *plan, const void *const *shard_span_ptrs, uint32_t k,
                           uint32_t lost, const void *parity_dev, void *const *out_span_ptrs,
                           reft_stream stream);

/* ---- rotated placement of the parity (section 4.2, AEC) -------------------------------------------
 * The paper's layout of the redundancy: each of the k members of a group cuts its shard into k-1
 * segments of Lseg = ceil(L / (k-1)) bytes (the last one zero-extended) and stores the parity of
 * ONE segment of every OTHER member, so that every segment of every shard is protected exactly
 * once and each member holds shard / (k-1) bytes of redundancy (the paper's W_n / (m (m-1))).
 * Member i protects, from shard j != i, segment r(i, j) = i if i < j, else i - 1; for the first
 * member this is Eq. 1 literally (p_bcd0 = b_0 xor c_0 xor d_0).  The figure that shows the
 * layout for the other members is not available; this is the reading taken.
 *
 * reft_segment_bytes            Lseg for this plan and k (0 if k < 2).
 * reft_parity_encode_rotated    parity_dev[0..Lseg) = XOR over j != member of segment r(member, j)
 *                               of shard j, read in place through the span pointers (row `member`
 *                               of shard_span_ptrs is ignored).
 * reft_reconstruct_rotated      decodes the lost member's shard into out_span_ptrs, segment by
 *                               segment (Eq. 2): segment r is protected by the member i with
 *                               r(i, lost) = r and equals parity_ptrs[i] xor the other segments
 *                               that unit covers.  Row `lost` of shard_span_ptrs and entry `lost`
 *                               of parity_ptrs are ignored (they were on the lost node);
 *                               parity_ptrs[i] are device pointers to Lseg bytes each.
 * 2 <= k <= REFT_MAX_K.  The first call for a given (k, member) or (k, lost) builds and caches
 * derived tables in the plan (allocates); later calls do not.
 * Errors: REFT_EINVAL (k, member or lost out of range, null pointers), REFT_EHIP.
 */
uint64_t reft_segment_bytes(const reft_plan *plan, uint32_t k);
int reft_parity_encode_rotated(reft_plan *plan, const void *const *shard_span_ptrs, uint32_t k,
                               uint32_t member, void *parity_dev, reft_stream stream);
int reft_reconstruct_rotated(reft_plan *plan, const void *const *shard_span_ptrs,
                             const void *const *parity_ptrs, uint32_t k, uint32_t lost,
                             void *const *out_span_ptrs, reft_stream stream);

/* ---- several redundancy strategies at once (section 4.2, Collaborative Redundant Protection) -------
 * The paper lets several strategies protect a group together - redundant copies (ARC: member i
 * also snapshots the shard of member (i + d) mod k; one strategy per offset d) and the rotated
 * parity units (AEC) - and states that N strategies survive N lost members.  What survives a given
 * loss depends on where the redundancy lay, so the library plans the recovery from the set of lost
 * members (host integer logic, no GPU needed); the steps themselves are the ordinary calls:
 *   REFT_RECOVER_COPY    reft_restore of the duplicate of `member`'s shard that surviving member
 *                        `source` keeps under copy_offsets[which];
 *   REFT_RECOVER_DECODE  reft_reconstruct_rotated of `member` from all other members' shards and
 *                        parity units.  Possible only when `member` is the only one lost: a second
 *                        lost member takes along the unit that covers one of its segments.
 * A lost member with a surviving duplicate is copied (the cheaper step); two redundant copies with
 * different offsets survive any two losses for k >= 3, while a copy plus the parity units survive
 * two losses only if neither lost member kept the other's duplicate.
 *
 * k             members of the group, 2 <= k <= REFT_MAX_K.
 * copy_offsets  n_copies offsets d, 1 <= d < k (may be NULL with n_copies == 0).
 * parity_units  non-zero if every member also keeps its rotated parity unit.
 * lost[k]       1 = member lost.
 * steps         receives one step per recoverable lost member, in member order (room for k).
 * nsteps        receives their number.
 * Returns REFT_OK if every lost member is recoverable, REFT_EUNRECOVERABLE if some are not (the
 * steps of those that are still come back), REFT_EINVAL for bad arguments.
 */
#define REFT_RECOVER_COPY   1
#define REFT_RECOVER_DECODE 2
typedef struct reft_recovery_step {
    uint32_t member;   /* the lost member this step recovers                                     */
    uint32_t how;      /* REFT_RECOVER_COPY or REFT_RECOVER_DECODE                                */
    uint32_t source;   /* COPY: the surviving member that keeps the duplicate                    */
    uint32_t which;    /* COPY: index into copy_offsets of the strategy the duplicate belongs to */
} reft_recovery_step;
int reft_recovery_plan(uint32_t k, const uint32_t *copy_offsets, uint32_t n_copies,
                       int parity_units, const uint8_t *lost, reft_recovery_step *steps,
                       uint32_t *nsteps);

/* ---- S5 + S7: load a shard from pinned host memory back into its tensors (section 4.3, step 1) ---
 * The inverse of reft_snapshot_pack, with the same two transports: staged (staging != NULL:
 * large pieces by hipMemcpyAsync on copy_stream straight into their tensors, runs of small pieces
 * by hipMemcpyAsync into a staging slot and a scatter kernel on unpack_stream) or direct (staging == NULL: the scatter kernel reads the pinned host snapshot
 * across the link, per bucket, on unpack_stream).  host_bytes must equal L (REFT_ESIZE).  Other
 * arguments as for reft_snapshot_pack.
 */
int reft_restore(reft_plan *plan, const void *host_src, uint64_t host_bytes,
                 void *staging, uint64_t staging_bytes,
                 void *const *span_ptrs, reft_stream copy_stream, reft_stream unpack_stream);
int reft_restore_wait(reft_plan *plan);

/* ---- tuning and diagnostics -----------------------------------------------------------------------
 * Process-wide launch parameters, read at each launch:
 *   "max_wgs"      cap on workgroups per kernel launch (0 = 16 per compute unit).  A small cap keeps
 *                  a snapshot kernel on few compute units while training kernels run beside it.
 *   "nontemporal"  1 = streaming (non-temporal) loads and stores in the kernels, 0 = plain.
 *   "unroll"       16-byte chunks in flight per thread and source: 1, 2 or 4.
 *   "link_wgs"     cap on workgroups of kernels bound by the host link (default 32; kernels
 *                  that read host memory use twice this).
 *   "dma_min_bytes"     staged transport: pieces of at least this size travel by DMA alone
 *                  (default 65536; 0 = every piece; a huge value = none, everything is gathered).
 *   "gather_min_pieces" staged transport: shortest run of smaller pieces that is gathered by a
 *                  kernel instead of being copied piece by piece (default 8, at least 1).
 *   "dma_streams"  staged transport: 1 (default) = all piece copies on copy_stream; 2 = they
 *                  alternate between copy_stream and a helper stream owned by the plan (forked from
 *                  and joined to copy_stream, default priority), which hides the set-up gap between
 *                  consecutive copies (56.2 -> 56.9 GB/s) - but only while the process has a free
 *                  hardware queue for it: with more streams than hardware queues (4 by default)
 *                  the helper shares a queue and transfers get slower instead.  The helper stream
 *                  is created with the plan if the tunable is 2 at that time, else by the first
 *                  call that wants it.
 *   "graph_copies" staged transport: 0 (default) = the piece copies are hipMemcpyAsync calls; 1 = they
 *                  are the independent memcpy nodes of a hipGraph that the plan builds once per
 *                  (tensors, host buffer, bucket range) and replays, 2 = the same as a chain of
 *                  nodes.  Fewer gaps between the copies of one snapshot (53.8 -> 55.6 GB/s), but two
 *                  such graphs on two streams do not overlap: use it where nothing else shares the
 *                  link in the other direction.
 *   "small_pieces" a tile in which at least this many spans start is processed by the LDS-staged
 *                  small-piece path of the gather / scatter kernels (default 8; 4294967295 = never,
 *                  0 = always).
 *   "burst"        1 (default) = reft_parity_encode, reft_reconstruct_spans and the rotated calls use
 *                  the write-burst variant of the XOR kernel where it applies: a pass (up to 8 rows
 *                  each) of at least "burst_min_rows" rows (default 5), "burst_min_bytes" stream
 *                  bytes (default 8 MiB), at most one tile in a hundred dense in small spans (see
 *                  "small_pieces"), and, for a decode into tensors, every tensor's address aligned
 *                  alike (mod 16) relative to its stream offset; reft_reconstruct uses it under
 *                  the first two conditions.  The variant keeps reads and writes apart in time: reader
 *                  waves XOR "burst_stage_bytes" (default 32768; a multiple of 4096, at most 65536)
 *                  of the stream at a time into LDS, and one writer wave per workgroup stores the
 *                  previous stage once all workgroups of the (persistent, "burst_wgs_per_cu" per
 *                  compute unit, default 2) grid have read theirs.  The writer waits by polling a
 *                  counter at most "burst_max_polls" times per round (default 6; 0 = never waits),
 *                  "burst_nap" x 1024 cycles apart (default 16); a writer whose wait runs out
 *                  does not wait at all for the next 1, 2, 4, ... 64 rounds.  Timing only: results
 *                  never depend on it.  0 = always the ordinary kernel.
 * Read when a plan is created:
 *   "tile_shift"   log2 of the tile size in bytes, 12..24 (default 18 = 256 KiB).
 *   "host_only_plans"  1 = reft_plan_create builds only the host-side sizing (no GPU needed);
 *                  such a plan answers the reft_plan_* queries and is refused (REFT_EINVAL) by
 *                  every call that would touch the GPU.
 * reft_set_tunable returns REFT_EINVAL for an unknown name or a value out of range.
 *
 * reft_plan_burst_stats (a diagnostic; waits for the device): how the writer waves of the plan's
 * most recent write-burst launch spent their rounds, summed over the workgroups: stats[0] rounds
 * in which the chip-wide meeting was seen complete, stats[1] rounds in which the polls ran out,
 * stats[2] rounds without waiting (back-off after a time-out), stats[3] group completions counted
 * by the meeting counter.  All zero if the plan has launched no burst kernel (or "burst_max_polls"
 * is 0).
 */
int reft_plan_burst_stats(reft_plan *plan, uint64_t stats[4]);
int reft_set_tunable(const char *name, uint64_t value);
int reft_get_tunable(const char *name, uint64_t *value);
const char *reft_last_error(void);   /* thread-local, never NULL */
const char *reft_version(void);

#ifdef __cplusplus
}
#endif
#endif /* REFT_H */
