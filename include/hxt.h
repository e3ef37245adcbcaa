/*
 * hxt.h -- C ABI of the per-GPU side of pipeline-parallel stage-boundary
 * transfers (activations forward, activation gradients backward) on MI355X.
 *
 * The operation follows the paper's Section 2.2 ("CPU-offloading P2P
 * mechanism"): the sender copies the user tensor device-to-device into a chunk
 * buffer, the chunk buffer is shipped, the receiver copies it symmetrically into
 * its own tensor.  Section 2.1 adds multi-NIC parallel transfer (here: k lanes)
 * and the CPU-forwarding variant with explicit GPU<->CPU buffer copies around
 * the wire.  The wire itself is not part of this library: on one GPU the packed
 * buffer written by hxt_pack (or refilled by hxt_stage_h2d) is the one
 * hxt_unpack reads.
 *
 * Layout contract (the paper fixes no constants; these are this library's):
 *   - Logical stream: tensors in order, each in row-major order of its shape
 *     (last index fastest) whatever its strides; every tensor starts at a
 *     multiple of 256 bytes and the stream length L is rounded up to 256; the
 *     gaps are zero.  message_bytes N = sum of tensor bytes.
 *   - Chunk c = stream bytes [c*chunk_bytes, min((c+1)*chunk_bytes, L)).
 *   - lane(c) = c mod n_lanes, slot(c) = c div n_lanes (round-robin).
 *   - Packed buffer, lane-major: lane l's region starts where lane l-1's ends
 *     and holds its chunks in slot order, chunk_bytes per slot;
 *     packed_bytes = num_chunks * chunk_bytes.  Slot bytes past a short last
 *     chunk are never read or written.
 *   - Checksum of chunk c = sum of its little-endian 32-bit words mod 2^64,
 *     taken over the chunk's padded length (pad bytes are zero).
 *
 * Conventions
 *   - Every function returns HXT_OK (0) or a negative hxt_status; nothing is
 *     written to outputs on error.  No function throws or aborts.
 *   - "device" pointers are HIP device addresses on the current device, "host"
 *     pointers ordinary process memory, "pinned" host memory from hipHostMalloc.
 *     A plan belongs to the device that was current when it was created; a
 *     data-plane call made with another device current returns HXT_EHIP.
 *   - The caller owns every data buffer and every stream.  The library owns only
 *     the plan (host tables plus one small device copy of its work tables,
 *     allocated by hxt_plan*, released by hxt_plan_destroy).
 *   - Data-plane calls only enqueue work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return; they never synchronise.
 *     Ordering between streams is the caller's business (events).
 *   - A plan's tables are immutable after creation and it may be used from
 *     several threads and streams.  Calls that ask for checksums use per-plan,
 *     per-operation accumulators: such calls on one stream are ordered by the
 *     stream, and when consecutive calls come on different streams the library
 *     makes the later stream wait for the earlier one (an event), so they never
 *     overlap; the claim of the accumulators and the enqueue of the kernels that
 *     use them are one critical section, so this also holds between threads.
 *     The sets are: hxt_pack; hxt_unpack and hxt_unpack_accumulate; hxt_checksum;
 *     hxt_checksum2, hxt_seal and hxt_pack_seal; hxt_verify and hxt_unpack_verify.
 *     One plan can therefore serve a sending stream and a receiving stream at the
 *     same time; messages that should overlap within one set need a plan each.
 *     The library remembers the stream that used a set last (it records the ordering
 *     event on it when the next call comes on another stream): a stream that has been
 *     given to such a call must stay alive until the plan is destroyed or until a later
 *     call of the same set has been made on another stream.
 *   - Stream capture: hxt_pack, hxt_unpack, hxt_unpack_accumulate, the batched calls,
 *     the checksum / seal / verify passes and the fused tag calls may be captured into a
 *     HIP graph (they record kernels only, no memset and no copy).  A call that asks for
 *     checksums and finds its accumulator set last used on another stream inserts the
 *     ordering event described above; make the first such call on the capture stream
 *     before capture begins, so that none is needed inside the graph.  A replayed graph
 *     keeps using the same accumulator set: do not run it concurrently with other calls
 *     of that set on the same plan.
 *   - Plans built from equal arguments on the sending and on the receiving side
 *     are interchangeable (the receive is symmetric).
 */
#ifndef HXT_H
#define HXT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HXT_MAX_DIMS 8
#define HXT_ALIGN 256 /* tensor starts, stream end, chunk_bytes, packed/pinned base pointers */

typedef enum {
    HXT_OK = 0,
    HXT_EINVAL = -1,       /* NULL where a pointer is required, bad count, bad lane, bad dtype ... */
    HXT_EALIGN = -2,       /* packed/pinned pointer not 256-byte aligned, tensor base not element aligned */
    HXT_EUNSUPPORTED = -3, /* valid request this library cannot serve (size limits) */
    HXT_EOVERLAP = -4,     /* hxt_unpack into a view whose elements may alias each other */
    HXT_EHIP = -5,         /* a HIP runtime call failed; hxt_last_hip_error() has the code */
    HXT_ENOMEM = -6        /* host or device allocation for the plan failed */
} hxt_status;

/* Only the element size matters to the transfer: data is moved as raw bits. */
typedef enum { HXT_U8 = 1, HXT_F16 = 2, HXT_BF16 = 3, HXT_F32 = 4, HXT_F64 = 5 } hxt_dtype_t;

typedef struct hxt_plan hxt_plan_t; /* opaque */

/* One tensor of a multi-tensor message.  strides in elements, NULL = contiguous. */
typedef struct {
    int ndim;               /* 0..HXT_MAX_DIMS */
    const int64_t *shape;   /* [ndim], each >= 0 */
    const int64_t *strides; /* [ndim], each >= 0, or NULL */
    hxt_dtype_t dtype;
} hxt_tensor_desc_t;

typedef struct {
    int32_t lane;        /* c mod n_lanes */
    int32_t slot;        /* c div n_lanes */
    uint64_t stream_off; /* c * chunk_bytes */
    uint64_t padded;     /* bytes of the chunk in the stream (multiple of 256) */
    uint64_t payload;    /* tensor bytes among them */
    uint64_t packed_off; /* where the chunk starts in the packed buffer */
} hxt_chunk_info_t;

typedef struct {
    uint64_t packed_off; /* start of the lane's region in the packed buffer */
    uint64_t bytes;      /* used bytes: up to the padded end of the lane's last chunk */
    int32_t n_chunks;
} hxt_lane_info_t;

/* ---- step 1: plan (host; Section 2.2: control work stays on the CPU) -------
 * Validates the geometry, merges dimensions that are contiguous in memory, cuts
 * the logical stream into chunks, deals the chunks over the lanes and builds the
 * device work tables.  Needs a GPU only for the device copy of those tables; with
 * no HIP device present the plan is still created and answers every query, and
 * the data-plane calls return HXT_EHIP.
 * Rejects with HXT_EINVAL: out == NULL, shape == NULL with ndim > 0, ndim < 0 or
 * > HXT_MAX_DIMS, a negative extent or stride, unknown dtype, n_lanes < 1 or
 * > 1024, chunk_bytes == 0 or not a multiple of 256, n_tensors < 0.
 * HXT_EUNSUPPORTED: message larger than 2^40 bytes, more than 2^31 chunks, or a view
 * whose farthest element lies 2^62 bytes or more past its base. */
int hxt_plan(const int64_t *shape, const int64_t *strides, int ndim, hxt_dtype_t dtype,
             int n_lanes, size_t chunk_bytes, hxt_plan_t **out);
int hxt_plan_multi(const hxt_tensor_desc_t *tensors, int n_tensors,
                   int n_lanes, size_t chunk_bytes, hxt_plan_t **out);
int hxt_plan_destroy(hxt_plan_t *plan); /* NULL is allowed */

/* ---- per-plan options (host only; not in the paper: tuning switches of this library) --
 * HXT_OPT_PACKED_HINT: cache hint of the packed-buffer side of every copy and pass of this plan.
 *   -1 (default) by size: cacheable while packed_bytes <= 128 MiB, so that a packed buffer that is
 *      re-read soon (by the wire, or by hxt_unpack on the same GPU) can be served from the 256 MB
 *      last-level cache; non-temporal above;
 *    0 always cacheable;  1 always non-temporal (every byte goes to and comes from HBM).
 *   The environment variable HXT_NT_PACKED (0/1), read when a plan is created, sets the initial value.
 *   Exception: the slower kernel variants taken when a tensor's base pointer is not 16-byte aligned
 *   keep both sides cacheable whatever the hint.
 * HXT_OPT_STAGE_D2H: how hxt_stage_d2h* and the CPU-forwarding path of hxt_exchange_stream move
 *   the packed buffer to pinned host memory.
 *    0 (default) a copy command (hipMemcpyAsync: the runtime picks a DMA engine or a blit kernel of
 *      its own, depending on what is outstanding when the call is made);
 *    1 the library's copy kernel (64 workgroups that store straight into the pinned buffer; the host
 *      buffer must then be device-accessible pinned memory, which hipHostMalloc memory is).  Same
 *      rate alone (55 GB/s); beside a host-to-device DMA copy it reaches 44 GB/s per direction where
 *      two DMA engines reach 49.
 *   Host-to-device staging always uses a copy command (a DMA engine).
 * Options take effect for calls made afterwards; do not change them while calls on the plan are being
 * issued from other threads.  HXT_EINVAL for an unknown option or value. */
typedef enum { HXT_OPT_PACKED_HINT = 1, HXT_OPT_STAGE_D2H = 2 } hxt_option_t;
int hxt_plan_set_option(hxt_plan_t *plan, int option, int value);

/* ---- queries (host only; not in the paper: what a caller needs to size its buffers and to
 * check the layout contract stated at the top of this file) -------------------------- */
size_t hxt_plan_message_bytes(const hxt_plan_t *plan); /* N */
size_t hxt_plan_stream_bytes(const hxt_plan_t *plan);  /* L */
size_t hxt_plan_packed_bytes(const hxt_plan_t *plan);  /* num_chunks * chunk_bytes */
size_t hxt_plan_chunk_bytes(const hxt_plan_t *plan);
int hxt_plan_num_chunks(const hxt_plan_t *plan);
int hxt_plan_num_lanes(const hxt_plan_t *plan);
int hxt_plan_num_tensors(const hxt_plan_t *plan);
int hxt_plan_chunk_info(const hxt_plan_t *plan, int c, hxt_chunk_info_t *out);
int hxt_plan_lane_info(const hxt_plan_t *plan, int lane, hxt_lane_info_t *out);
/* 1 if hxt_unpack may write through tensor t's view (no two elements alias), else 0 */
int hxt_plan_tensor_unpack_safe(const hxt_plan_t *plan, int t);
/* which kernel family serves tensor t: 0 none (empty), 1 contiguous copy, 2 row gather (runs and
 * pitches that are multiples of 16 bytes), 3 LDS transpose, 4 per-element, 6 row gather in narrower
 * pieces (runs of 16 bytes or more whose length or pitch is not a multiple of 16), 7 LDS transpose
 * whose tiles span chunks (a chunk holds fewer rows of the packed side than a tile is high) */
int hxt_plan_tensor_kind(const hxt_plan_t *plan, int t);

/* ---- step 2: pack (Section 2.2: user buffer -> chunk buffer, device to device)
 * src: host array of n_tensors device base pointers (element aligned; a tensor
 *   whose base is not 16-byte aligned is served by the same kernel with narrower
 *   accesses on its side).
 * packed: device, >= packed_bytes, 256-byte aligned.  Every chunk's padded bytes
 *   are written (pad = 0); nothing else.
 * sums: NULL, or device array of num_chunks uint64 that receives the send-side
 *   checksums of what was written (fused into the copy; no extra pass). */
int hxt_pack(const hxt_plan_t *plan, const void *const *src, void *packed,
             uint64_t *sums, void *stream);

/* ---- step 3: CPU-forwarding staging (Section 2.1: explicit GPU<->CPU copies) -
 * Copies the used bytes of one lane (lane >= 0) or of all lanes (lane == -1)
 * between the device packed buffer and a pinned host buffer of the same layout
 * (same offsets).  Both buffers >= packed_bytes and 256-byte aligned. */
int hxt_stage_d2h(const hxt_plan_t *plan, int lane, const void *packed_dev,
                  void *host_pinned, void *stream);
int hxt_stage_h2d(const hxt_plan_t *plan, int lane, const void *host_pinned,
                  void *packed_dev, void *stream);

/* The same for a run of slots of one lane: slots [first_slot, first_slot + n_slots) of lane `lane`
 * (slot s of lane l holds chunk s * n_lanes + l), each up to its chunk's padded end, so that a lane
 * can be staged in pieces and the two directions pipelined chunk by chunk.  HXT_EINVAL if lane < 0
 * or the run reaches past the lane's last chunk; n_slots == 0 is a no-op. */
int hxt_stage_d2h_slots(const hxt_plan_t *plan, int lane, int first_slot, int n_slots,
                        const void *packed_dev, void *host_pinned, void *stream);
int hxt_stage_h2d_slots(const hxt_plan_t *plan, int lane, int first_slot, int n_slots,
                        const void *host_pinned, void *packed_dev, void *stream);

/* ---- widening of step 3: the host-side hop of the CPU-forwarding path ------------
 * Section 2.1: in the compatibility path the data travels between the two hosts through
 * a CPU-side transport, one NIC per lane.  On one machine that hop is a host-to-host
 * copy from the pinned buffer device-to-host staging filled into the pinned buffer
 * host-to-device staging reads, lane by lane on parallel threads.
 *   hxt_host_forward: synchronous, pure host (no GPU needed).  Copies the used bytes of
 *     lane `lane` (or of every lane, lane == -1) from `from` to `to` at the same offsets,
 *     with up to n_threads threads (one lane per thread at a time; n_threads < 1 = one per
 *     lane; never more than 64, the calling thread included; if a thread cannot be started its
 *     lanes are copied by the calling thread).  Both buffers >= packed_bytes; they must not overlap.
 *   hxt_stage_hop: the same copy enqueued on `stream` (it runs on a host thread once the
 *     work enqueued before it has finished, and later work on the stream waits for it).
 * HXT_EINVAL for NULL buffers or a bad lane. */
int hxt_host_forward(const hxt_plan_t *plan, int lane, const void *from, void *to, int n_threads);
int hxt_stage_hop(const hxt_plan_t *plan, int lane, const void *from_pinned, void *to_pinned,
                  int n_threads, void *stream);

/* ---- step 4: unpack (Section 2.2: the receiver's symmetric copy) -------------
 * dst: host array of n_tensors device base pointers.  Writes exactly the bytes
 * the views address.  HXT_EOVERLAP if some tensor's view is not unpack-safe.
 * sums: NULL, or device array receiving the receive-side checksums of the packed
 * bytes as read (pad included). */
int hxt_unpack(const hxt_plan_t *plan, const void *packed, void *const *dst,
               uint64_t *sums, void *stream);

/* ---- widening of step 4: receive and accumulate --------------------------------
 * Section 2.2: the intermediate results of each vendor's local reduction cross the
 * boundary by the same P2P mechanism and are combined on arrival.  Like hxt_unpack,
 * but every destination element becomes old + arriving instead of being overwritten:
 *   HXT_BF16: both operands widened exactly to binary32, added in binary32 (round to
 *             nearest even), the sum rounded to bf16 to nearest, ties to even;
 *   HXT_F32 : IEEE binary32 addition.
 * A NaN result is stored as the canonical quiet NaN (0x7FC0 / 0x7FC00000).
 * Supported for plans whose non-empty tensors are all contiguous and of those two
 * dtypes (HXT_EUNSUPPORTED otherwise); destinations element aligned, as in hxt_unpack.
 * sums: as in hxt_unpack (checksums of the packed bytes as read). */
int hxt_unpack_accumulate(const hxt_plan_t *plan, const void *packed, void *const *dst,
                          uint64_t *sums, void *stream);

/* The same for n messages at once, like hxt_unpack_batch: messages that are one contiguous
 * 16-byte aligned tensor each share kernel launches (up to 4 per launch), the others are
 * enqueued one by one; results are those of n hxt_unpack_accumulate calls.  sums: NULL, or an
 * array of n entries each NULL or a device array of that plan's num_chunks values; a plan may
 * appear twice only if at most one of its entries asks for sums (HXT_EINVAL otherwise).
 * Everything is validated before anything is enqueued. */
int hxt_unpack_accumulate_batch(int n, const hxt_plan_t *const *plans, const void *const *packed,
                                void *const *const *dst, uint64_t *const *sums, void *stream);

/* ---- steps 2 and 4 for several messages at once -------------------------------
 * A stage boundary is crossed in both directions at the same point of the schedule
 * (Section 3.1: two pipeline stages; the forward activation of one micro-batch and
 * the backward gradient of another).  These calls take n independent messages, each
 * with its own plan, tensors, packed buffer and (optional) checksum array, and give
 * exactly the result of n hxt_pack / hxt_unpack calls on `stream` in order, but
 * messages that consist of one contiguous 16-byte aligned tensor share kernel
 * launches (up to 4 per launch), which removes per-launch ramp-up for small messages.
 * plans[i], src[i] / dst[i] (array of that plan's tensor pointers) and packed[i] as
 * in the single-message calls; sums may be NULL, and sums[i] may be NULL.
 * HXT_EINVAL additionally if one plan appears twice with checksums requested (its
 * accumulators serve one message at a time).  Nothing is enqueued on error. */
int hxt_pack_batch(int n, const hxt_plan_t *const *plans, const void *const *const *src,
                   void *const *packed, uint64_t *const *sums, void *stream);
int hxt_unpack_batch(int n, const hxt_plan_t *const *plans, const void *const *packed,
                     void *const *const *dst, uint64_t *const *sums, void *stream);

/* ---- step 6: a stream of micro-batches through ping-pong buffers ----------------
 * Enqueues pack -> (staging) -> unpack for n_messages messages of one geometry so that
 * the steps of consecutive messages overlap: message i uses buffer set i mod n_buffers;
 * pack runs on stream_pack, the device-to-host copies on stream_stage, the
 * host-to-device copies and unpack on stream_unpack; events owned by the plan (created the
 * first time they are needed, released by hxt_plan_destroy) order
 * them (pack of message i waits until buffer set i mod n_buffers has been drained by
 * message i - n_buffers, and so on).  This is the host-side event-handling half of
 * Section 2.2's control plane for a 1F1B schedule, where a stage sends one micro-batch
 * while the previous one is still in flight.
 *   path HXT_DEVICE_DIRECT: unpack reads packed_send[b] (packed_recv, host_pinned unused).
 *       Which stream runs what is then chosen by direct_mode, the results and the
 *       completion rule below being the same:
 *       HXT_DIRECT_TWO_CHAINS  even messages are packed and unpacked on stream_pack and odd
 *           messages on stream_unpack (two independent chains whose kernels overlap, no events
 *           inside); needs an even n_buffers and distinct stream_pack / stream_unpack.  This
 *           is loopback-shaped: a message is unpacked right behind its own pack.
 *       HXT_DIRECT_FUSED  launches on stream_pack that unpack message i-1 and pack message i
 *           together; needs n_buffers >= 2, single-tensor 16-byte aligned messages, no tags.
 *       HXT_DIRECT_EVENTS  pack on stream_pack, unpack on stream_unpack after an event, as at
 *           a real boundary where the unpack waits for the arrival; any message.
 *       HXT_DIRECT_AUTO  the first of the three, in that order, that the arguments allow.
 *   path HXT_CPU_FORWARD  : packed_send[b] -> host_pinned[b] -> packed_recv[b] -> unpack.
 * src/dst: n_messages * n_tensors device pointers, message-major.  send_sums/recv_sums:
 * NULL or device arrays of n_messages * num_chunks uint64, message-major.
 * The call only enqueues and never waits on the host, unless the caller asks for it with
 * drain_every > 0 (HXT_CPU_FORWARD only): the call then waits for the three streams to run empty
 * after every drain_every messages.  That is a workaround for the HIP runtime on this machine,
 * which stops overlapping the two copy directions once more than about 16 messages' worth of copies
 * and event waits are outstanding (12 is the measured best); such a call blocks the calling thread
 * and must not be made under stream capture.  With drain_every == 0 a caller can get the same
 * effect without blocking inside the library by issuing the stream in windows of its own
 * (n_messages <= 12 per call, waiting for the streams between calls).  When the three streams have
 * drained, every message has arrived.
 * HXT_EINVAL: n_messages < 0, n_buffers < 1, drain_every < 0, an unknown direct_mode or one that the
 * arguments do not allow, a NULL array that the path needs;
 * a NULL stream handle shared by two roles is allowed (the steps then serialise). */
typedef enum { HXT_DEVICE_DIRECT = 0, HXT_CPU_FORWARD = 1 } hxt_path_t;
typedef enum { HXT_DIRECT_AUTO = 0, HXT_DIRECT_TWO_CHAINS = 1, HXT_DIRECT_FUSED = 2, HXT_DIRECT_EVENTS = 3 } hxt_direct_mode_t;

typedef struct {
    int n_messages;
    int n_buffers;
    hxt_path_t path;
    const void *const *src;    /* [n_messages * n_tensors] */
    void *const *dst;          /* [n_messages * n_tensors] */
    void *const *packed_send;  /* [n_buffers] device, >= packed_bytes, 256-byte aligned */
    void *const *packed_recv;  /* [n_buffers] device (CPU forwarding) */
    void *const *host_pinned;  /* [n_buffers] pinned host (CPU forwarding) */
    uint64_t *send_sums;       /* device, n_messages * num_chunks, or NULL */
    uint64_t *recv_sums;       /* device, n_messages * num_chunks, or NULL */
    void *stream_pack;
    void *stream_stage;
    void *stream_unpack;
    /* Optional chunk tags (see hxt_seal / hxt_verify below): tags_send == NULL = none.  With
     * tags, message i is sealed with seq = seq_base + i and micro_batch = i inside its pack, the
     * tags travel with the message (through tags_pinned on the CPU-forwarding path) and are
     * verified inside its unpack; send_sums / recv_sums must then be NULL (HXT_EINVAL). */
    void *const *tags_send;    /* [n_buffers] device, num_chunks * 64 bytes, 16-byte aligned */
    void *const *tags_recv;    /* [n_buffers] device (CPU forwarding) */
    void *const *tags_pinned;  /* [n_buffers] pinned host (CPU forwarding) */
    uint32_t *status;          /* device, n_messages * (num_chunks + 1): hxt_verify's result per message */
    uint64_t seq_base;
    int direct_mode;           /* hxt_direct_mode_t; HXT_DEVICE_DIRECT only */
    int drain_every;           /* 0 = enqueue only; > 0: wait on the host after every so many messages (HXT_CPU_FORWARD) */
} hxt_exchange_t;

int hxt_exchange_stream(const hxt_plan_t *plan, const hxt_exchange_t *x);

/* ---- step 5: stand-alone per-chunk checksum of a packed buffer (not in the paper: the
 * integrity check of this library's contract, also available fused into hxt_pack /
 * hxt_unpack through their `sums` argument) ------------------------------------------ */
int hxt_checksum(const hxt_plan_t *plan, const void *packed, uint64_t *sums, void *stream);

/* ---- widening of step 5: a check that also sees words that changed places --------
 * The plain sum is blind to a permutation of words inside a chunk.  For chunk c with
 * words w_0 .. w_{W-1} this writes sums2[2c] = sum_j w_j and sums2[2c+1] =
 * sum_j (j+1) * w_j, both mod 2^64 (swapping words i and j changes the second by
 * (j-i) * (w_i - w_j) != 0).  Stand-alone pass over a packed buffer (reads N bytes).
 * sums2: device array of 2 * num_chunks uint64. */
int hxt_checksum2(const hxt_plan_t *plan, const void *packed, uint64_t *sums2, void *stream);

/* ---- widening: chunk tags (subsection "Engineering Challenges": the hangs met while
 * bringing up the mixed-vendor transfer) -------------------------------------------
 * The paper defines no header; this one is this library's contract.  A tag says which
 * message and which chunk a packed slot holds and carries both sums, so that a stale
 * ping-pong buffer, a misrouted lane or damaged bytes are reported by the receiver
 * instead of being unpacked.  Tags are kept beside the packed buffer (its layout does
 * not change): one 64-byte record per chunk, in packed-slot order (the tag of chunk c
 * is number packed_off(c) / chunk_bytes, so a lane's tags are one contiguous run that
 * can travel with the lane).  All fields little-endian. */
typedef struct {
    uint32_t magic;        /* HXT_TAG_MAGIC */
    uint32_t chunk;        /* c */
    uint32_t lane, slot;   /* c mod k, c div k */
    uint64_t seq;          /* sender's running message number */
    uint32_t micro_batch;  /* sender's micro-batch id */
    uint32_t n_chunks;     /* C */
    uint64_t padded;       /* bytes of the chunk that are transferred */
    uint64_t sum;          /* as hxt_checksum2 */
    uint64_t wsum;
    uint64_t zero;
} hxt_chunk_tag_t;
#define HXT_TAG_MAGIC 0x31545848u /* bytes 'H','X','T','1' */

enum hxt_tag_status {            /* bits of a chunk's verification result, 0 = accepted */
    HXT_TAG_BAD_MAGIC = 1,
    HXT_TAG_BAD_PLACE = 2,       /* chunk, lane, slot, n_chunks or padded differ from the receiver's plan */
    HXT_TAG_BAD_SEQ = 4,
    HXT_TAG_BAD_MICRO_BATCH = 8,
    HXT_TAG_BAD_SUM = 16,        /* the received bytes do not add up to the tag's plain sum */
    HXT_TAG_BAD_WSUM = 32,       /* ... to its position-weighted sum */
    HXT_TAG_BAD_RESERVED = 64    /* last field not zero */
};

/* Sender: one pass over `packed` (reads N bytes) that writes the num_chunks tags.
 * tags: device, num_chunks * 64 bytes, 16-byte aligned (HXT_EALIGN otherwise). */
int hxt_seal(const hxt_plan_t *plan, const void *packed, uint64_t seq, uint32_t micro_batch,
             hxt_chunk_tag_t *tags, void *stream);

/* Receiver: one pass over the received `packed` that recomputes both sums of every
 * chunk and checks the tag found at the chunk's slot against the receiver's own plan,
 * the expected seq / micro_batch and the recomputed sums.
 * status: device, num_chunks + 1 uint32; status[c] = OR of hxt_tag_status bits for chunk
 * c, status[num_chunks] = number of chunks with a non-zero mask (written by the workgroup
 * that completes the last chunk).  The caller reads status back and decides;
 * nothing is compared on the host by the library. */
int hxt_verify(const hxt_plan_t *plan, const void *packed, const hxt_chunk_tag_t *tags, uint64_t seq,
               uint32_t micro_batch, uint32_t *status, void *stream);

/* The same, fused into the copies (no extra pass over the message when all its tensors
 * are contiguous and 16-byte aligned: one activation, or a bucket of gradients; otherwise
 * the two passes run one after the other on the stream, with identical results):
 * hxt_pack_seal = hxt_pack + hxt_seal,
 * hxt_unpack_verify = hxt_verify + hxt_unpack.  The destination is written whatever the
 * verdict; the caller reads `status` before using it.  Arguments as in those calls. */
int hxt_pack_seal(const hxt_plan_t *plan, const void *const *src, void *packed, uint64_t seq,
                  uint32_t micro_batch, hxt_chunk_tag_t *tags, void *stream);
int hxt_unpack_verify(const hxt_plan_t *plan, const void *packed, const hxt_chunk_tag_t *tags,
                      uint64_t seq, uint32_t micro_batch, void *const *dst, uint32_t *status,
                      void *stream);

/* ---- for callers that cannot allocate ----------------------------------------------
 * Code under HIP graph capture, tight serving loops and harnesses that forbid allocation
 * cannot create a plan (hxt_plan* allocates device memory).  hxt_pack_noalloc is hxt_pack for
 * a message that is ONE contiguous tensor of message_bytes bytes at `src` (device, any
 * alignment; 16-byte aligned is the fast path), with the same layout contract, the same
 * packed bytes and the same checksums as hxt_pack on hxt_plan({message_bytes}, NULL, 1,
 * HXT_U8, n_lanes, chunk_bytes).  It needs no plan, and neither it nor anything it calls
 * allocates host or device memory: the geometry is computed on the stack, and the checksum
 * accumulators live in a fixed 1 MiB device array that is part of the library image (each
 * GPU the library runs on holds its copy until the process ends).
 *   packed: device, >= ceil(L / chunk_bytes) * chunk_bytes with L = message_bytes rounded up
 *           to 256; 256-byte aligned.
 *   sums:   NULL, or device array of ceil(L / chunk_bytes) uint64.
 * Limit: with checksums, num_chunks * (f + 1) <= 4096, where f = 1 for chunks of fewer than
 * 128 tiles of 16 KiB (chunk_bytes < 2 MiB), else the largest power of two <= min(16,
 * tiles per chunk / 64); HXT_EUNSUPPORTED beyond (nothing is enqueued).  Other errors as
 * hxt_plan / hxt_pack.  message_bytes == 0 is a no-op.
 * All calls on one GPU share that array (the call zero-fills the part it uses, with a
 * kernel, on `stream` first): calls that ask for checksums and overlap in time on one GPU,
 * on different streams or from a replayed graph, race; order them.  The device address of
 * the array is looked up on the first call on each device: make that call before stream
 * capture begins. */
int hxt_pack_noalloc(const void *src, size_t message_bytes, int n_lanes, size_t chunk_bytes,
                     void *packed, uint64_t *sums, void *stream);

/* The fused tag calls for several messages at once, as hxt_pack_batch / hxt_unpack_batch are for
 * the plain sums: exactly the result of n hxt_pack_seal / hxt_unpack_verify calls on `stream` in
 * order; messages that consist of one contiguous 16-byte aligned tensor share launches (up to 4 per
 * launch).  seq[i], micro_batch[i], tags[i], status[i] belong to message i.  HXT_EINVAL also if a
 * plan appears twice.  Nothing is enqueued on error. */
int hxt_pack_seal_batch(int n, const hxt_plan_t *const *plans, const void *const *const *src,
                        void *const *packed, const uint64_t *seq, const uint32_t *micro_batch,
                        hxt_chunk_tag_t *const *tags, void *stream);
int hxt_unpack_verify_batch(int n, const hxt_plan_t *const *plans, const void *const *packed,
                            const hxt_chunk_tag_t *const *tags, const uint64_t *seq,
                            const uint32_t *micro_batch, void *const *const *dst,
                            uint32_t *const *status, void *stream);

/* ---- diagnostics -------------------------------------------------------------- */
const char *hxt_strerror(int status);
int hxt_last_hip_error(void);    /* hipError_t of the last failing HIP call on this thread */
const char *hxt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HXT_H */
