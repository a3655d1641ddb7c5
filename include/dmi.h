/*
 * dmi.h -- C ABI of the capture-and-stage library for model-internal
 * observability on AMD Instinct MI355X (gfx950).
 *
 * The library is the Ring^2 staging mechanism of the DMI-Lib paper (section 4.2)
 * together with the first stage of its data exporter (section 4.3) and the
 * policy manager's bandwidth controls (section 4.4), for one GPU:
 *
 *   producer   dmi_observe / dmi_observe_paged launch one HIP kernel on the
 *              caller's stream.  The kernel gathers the selected rows of the
 *              observed tensor, optionally downcasts them and reduces them to
 *              per-row summaries, and packs them behind a 64-byte descriptor
 *              into a byte ring in device memory.  The observed tensor is never
 *              modified and never retained (section 4.1).
 *   consumer   dmi_drain moves committed bytes into a pinned host ring;
 *              dmi_poll_host exposes whole records there; dmi_release_host
 *              gives the space back.
 *   policy     completeness (block), record-granular best effort (drop newest,
 *              counted), 1-in-k step sampling, per-point enable (hook filtering).
 *
 * Record layout in both rings (little endian, every pad byte zero; all sections
 * are padded to 64 bytes, so ring capacities and record sizes are multiples of 64
 * and a stream byte b lives at offset b mod capacity):
 *
 *   header 64 B : 0 u32 magic 0x32494D44 | 4 u16 version 1 | 6 u16 header_bytes 64
 *                 8 u64 seq | 16 u64 step_id | 24 u32 point_id
 *                 28 u8 src_dtype | 29 u8 out_dtype | 30 u8 summary_mask
 *                 31 u8 flags (DMI_REC_PAGED | DMI_REC_MASKED | DMI_REC_INDEXED)
 *                 32 u32 n_reqs | 36 u32 n_rows | 40 u32 row_elems | 44 u32 rank_tag
 *                 48 u64 record_bytes | 56 u64 payload_bytes
 *   req table   : n_reqs x { u32 req_id, u32 tok_start, u32 tok_step, u32 n_rows_r }
 *   payload     : n_rows x row_elems x sizeof(out_dtype), request-major, tokens
 *                 ascending, tightly packed (absent if out_dtype is DMI_DTYPE_NONE)
 *   summaries   : for each set bit of summary_mask in ascending order
 *                 (L2, mean, absmax): f32[n_rows]
 *
 * Conventions.  Pointers are marked [host] or [device].  The library owns both
 * rings; the caller owns every tensor, block table, mask and index list and
 * keeps them valid until the launched kernel has run on its stream.  No call
 * synchronises the caller's stream.  All observes of one ring must execute on
 * the GPU in call order (one stream, or streams chained by events).  One
 * producer thread per ring; dmi_drain / dmi_poll_host / dmi_release_host /
 * dmi_get_stats may be called from another thread.  Every function returns
 * DMI_OK (0), a positive informational code, or a negative error; after an
 * error dmi_last_error() gives a message (thread local).  Nothing throws.
 */
#ifndef DMI_H
#define DMI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dmi_ring dmi_ring_t;   /* opaque, library-owned */
typedef int32_t dmi_status_t;

enum {
    DMI_OK = 0,
    DMI_SAMPLED_OUT = 1,        /* step not selected by 1-in-k sampling: nothing captured */
    DMI_POINT_DISABLED = 2,     /* point switched off: nothing captured */
    DMI_ERR_INVALID_ARG = -1,
    DMI_ERR_NOMEM = -2,
    DMI_ERR_TOO_LARGE = -3,     /* the record can never fit the device ring (or the host ring) */
    DMI_ERR_HIP = -4,           /* a HIP call failed (also: no GPU present) */
    DMI_ERR_AGAIN = -5,         /* would block: no room and nothing more can be drained */
    DMI_ERR_CLOSED = -6
};

enum { DMI_DTYPE_NONE = 0, DMI_DTYPE_BF16 = 1, DMI_DTYPE_FP16 = 2, DMI_DTYPE_FP32 = 3,
       DMI_DTYPE_FP8_E4M3FN = 4 };
enum { DMI_SUM_L2 = 1, DMI_SUM_MEAN = 2, DMI_SUM_ABSMAX = 4 };
enum { DMI_REC_PAGED = 1, DMI_REC_MASKED = 2, DMI_REC_INDEXED = 4 };
enum { DMI_POLICY_BLOCK = 0, DMI_POLICY_DROP_NEWEST = 1 };

/* ring flags */
enum {
    DMI_DRAIN_COPY_ENGINE = 1,  /* drain with hipMemcpyAsync on a side stream (default) */
    DMI_DRAIN_KERNEL = 2,       /* drain with a copy kernel writing pinned host memory */
    DMI_BG_THREAD = 4           /* the library runs its own drain thread (section 4.3) */
};
/* dmi_drain flags */
enum {
    DMI_DRAIN_NONBLOCK = 1,     /* issue the copies and return without waiting for them */
    DMI_DRAIN_FLUSH = 2         /* first wait until every observe issued so far has committed */
};

#define DMI_MAGIC 0x32494D44u
#define DMI_HEADER_BYTES 64u
#define DMI_MAX_HEADS_SEL 8u
#define DMI_MAX_POINTS 4096u

/*
 * Ring creation (paper section 4.2: bounded staging, allocated once).
 *   device_ring_bytes, host_ring_bytes: capacities, multiples of 64, >= 4096.
 *   device_id: HIP device ordinal.   flags: ring flags above (0 = copy engine).
 *   max_reqs_per_observe: upper bound on n_reqs of any observe (0 = 1024, at most 4096:
 *             the per-request prefix sums live in LDS).
 *   rank_tag: written into every header (section 4.5: records carry the
 *             producer's parallel coordinates).
 *   bg_min_bytes, bg_min_records, bg_occupancy_pct, bg_timeout_us: when the library's drain
 *             thread issues a batch of copies (section 4.3: batched to avoid fragmented
 *             transfers, "once enough ready entries accumulate, or configurable occupancy,
 *             byte-count, or timeout thresholds are reached"): as soon as this many committed
 *             bytes are waiting, or this many committed records, or the device ring is this
 *             full (per cent of its capacity, undrained bytes), or the oldest waiting byte has
 *             waited this long.  0 = 1 MiB / 64 records / 50 % / 200 us.  A trigger is switched
 *             off by a value it cannot reach (UINT64_MAX, UINT32_MAX, more than 100, UINT32_MAX).
 *   block_timeout_ms: how long a blocking call waits for room before returning
 *             DMI_ERR_AGAIN (0 = 2000 ms).
 * Returns DMI_ERR_HIP if the device or a HIP allocation is not available,
 * DMI_ERR_INVALID_ARG for bad sizes.  *out is written only on success.
 */
typedef struct {
    uint64_t device_ring_bytes;
    uint64_t host_ring_bytes;
    int32_t device_id;
    uint32_t flags;
    uint32_t max_reqs_per_observe;
    uint32_t rank_tag;
    uint64_t bg_min_bytes;
    uint32_t bg_timeout_us;
    uint32_t block_timeout_ms;
    uint32_t bg_min_records;
    uint32_t bg_occupancy_pct;
} dmi_ring_config_t;

/* The environment variable DMI_DRAIN_MODE ("copy" or "kernel") overrides the drain engine chosen in flags. */
dmi_status_t dmi_ring_create(const dmi_ring_config_t *cfg /*[host]*/, dmi_ring_t **out /*[host]*/);

/* End of the staging rings' life (section 4.2: allocated once, for the whole run): stops the
 * drain thread and the exporter, waits for the library's own streams, frees both rings and the
 * control memory.  Undrained data is discarded.  The caller must have synchronised the streams
 * it passed to dmi_observe, and destroyed the ring's replayable steps. */
dmi_status_t dmi_ring_destroy(dmi_ring_t *ring);

/* Observed tensor: a row-major matrix [shape[0], shape[1]] of `dtype`
 * (BF16 / FP16 / FP32), stride in elements, stride[1] == 1.  Any 2-byte (4 for
 * FP32) aligned base and any shape are accepted; 16-byte aligned bases and row
 * pitches with shape[1]*sizeof(dtype) % 16 == 0 take the vectorised kernel. */
typedef struct {
    const void *data;           /* [device] */
    uint32_t dtype;
    int64_t shape[2];
    int64_t stride[2];
} dmi_tensor_t;

/* One request's token range.  Dense tensors: the j-th selected row (j < tok_count)
 * is tensor row  row_base + tok_start + j*tok_step.  Paged caches: row_base is the
 * request's row in the block table and tok_start + j*tok_step a logical token
 * position.  req_id, tok_start and tok_step are copied into the record's request
 * table (the metadata the paper keeps in its TensorMetaFIFO, section 4.2). */
typedef struct {
    uint32_t req_id, row_base, tok_start, tok_count, tok_step;
} dmi_req_sel_t;

/* Ragged per-request row selection.
 *   reqs          [host]   n_reqs entries, copied during the call.
 *   keep_mask_dev [device] optional, n_reqs bytes, read when the kernel runs:
 *                 request r is captured iff keep_mask_dev[r] != 0 (the paper's
 *                 batch-aligned keep/drop vector, section 4.4; it changes data,
 *                 not launch topology).
 *   row_index_dev [device] optional (dense only): explicit tensor row for every
 *                 listed row, request-major, sum(tok_count) int32 entries; masked-out
 *                 requests still occupy their entries.  tok_start/tok_step are then
 *                 metadata only. */
typedef struct {
    uint32_t n_reqs;
    const dmi_req_sel_t *reqs;
    const uint8_t *keep_mask_dev;
    const int32_t *row_index_dev;
} dmi_selection_t;

/* What is stored per row.  out_dtype: NONE (summaries only), the source dtype
 * (raw copy), or, from a BF16 source, FP16 or FP8_E4M3FN (round to nearest even;
 * FP8 saturates to +-448, NaN stays NaN).  summary_mask: DMI_SUM_* bits, fp32
 * reductions over the source row: L2 = sqrt(sum x^2), mean = sum x / row length,
 * absmax = max |x|; a row holding a NaN gives NaN for all three.
 * Limit of L2: the squares are summed in fp32, so a row whose sum of squares leaves
 * fp32's range gives +inf (some |x| beyond 1.8e19 / sqrt(how many such elements))
 * or 0 (every |x| below about 1e-22) although the norm itself is representable;
 * mean and absmax are exact in those cases. */
typedef struct {
    uint32_t out_dtype;
    uint32_t summary_mask;
} dmi_transform_t;

/*
 * Capture one tensor (paper section 4.2 step 1-2, section 4.4 gather-compact).
 * Launches one kernel on hip_stream [hipStream_t, 0 = null stream] and returns.
 * Policy: disabled point -> DMI_POINT_DISABLED; step_id % sample_k != sample_phase
 * -> DMI_SAMPLED_OUT; record larger than the device ring or the host ring -> DMI_ERR_TOO_LARGE;
 * DMI_POLICY_BLOCK with no room -> drains, waiting on the host up to
 * block_timeout_ms, then DMI_ERR_AGAIN; DMI_POLICY_DROP_NEWEST never waits: the
 * kernel discards the record if it does not fit when it runs, and counts it.
 * A sequence number is consumed only when a kernel is launched.
 * Besides the capture kernel the library puts small operations of its own on the stream
 * most recently passed here: an event every 16 launches or so, in best-effort mode (or with
 * keep vectors) also a one-workgroup launch that copies 64 bytes to pinned memory; dmi_drain
 * and the library's drain thread may add one when the producer has paused.  Do not capture
 * that stream into a graph by hand while captures are outstanding: use dmi_step_t.
 * Keep the stream alive until dmi_drain(DMI_DRAIN_FLUSH) has returned DMI_OK (or the ring
 * is destroyed) after the last observe on it.
 */
dmi_status_t dmi_observe(dmi_ring_t *ring, uint32_t point_id, const dmi_tensor_t *tensor /*[host]*/,
                         const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                         uint64_t step_id, void *hip_stream);

/* Paged KV cache: element (block b, slot s, head h, dim d) is at
 * base + b*block_stride + s*slot_stride + h*head_stride + d (strides in elements).
 * block_table_dev [device] int32 [n_seqs][block_table_stride]: physical block of
 * logical block t / block_size of a sequence.  A captured row is the
 * concatenation of head_dim elements of each selected head, in heads_sel order. */
typedef struct {
    const void *base;           /* [device] */
    uint32_t dtype;
    int64_t block_stride, slot_stride, head_stride;
    uint32_t block_size, n_heads, head_dim;
    uint32_t n_blocks;          /* physical blocks in the cache (bounds for table entries) */
    uint32_t n_seqs;            /* rows of the block table */
    const int32_t *block_table_dev;
    int64_t block_table_stride;
    uint32_t n_heads_sel;
    uint32_t heads_sel[DMI_MAX_HEADS_SEL];
} dmi_paged_kv_t;

/* As dmi_observe, for slices of a paged KV cache (the paper lists KV-cache
 * slices among the observable states, section 1; the block-table walk is this
 * build's).  sel->row_index_dev must be NULL. */
dmi_status_t dmi_observe_paged(dmi_ring_t *ring, uint32_t point_id, const dmi_paged_kv_t *kv /*[host]*/,
                               const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                               uint64_t step_id, void *hip_stream);

/*
 * Several observation points in one launch (paper section 5, "Device-to-device kernel": one
 * launch per observed tensor; a launch has a fixed cost of a few microseconds on the GPU, which
 * a decode step's small tensors cannot amortise one by one).  When n tensors of one dtype, shape
 * and stride are alive together and share selection and transform -- the residual stream of
 * every layer kept until the end of a decode step, K and V slices of several layers -- one
 * call captures them all:
 *   point_ids [host]  n observation points, one per tensor
 *   data      [host]  n [device] pointers: the tensors' data (dense) / the caches' bases (paged)
 *   like      [host]  dtype, shape and stride (dense) or the cache geometry, block table and
 *                     selected heads (paged) common to all of them; its data / base field is ignored
 * The result is, byte for byte and counter for counter, what n calls of dmi_observe /
 * dmi_observe_paged in array order would give with nothing happening between them: n records
 * with consecutive sequence numbers in array order (section 4.2: ring order is hook order), each
 * tensor passing hook filtering on its own (a disabled point is skipped and counted), sampling
 * applied to the step, drop-newest deciding per record (the records that still fit are kept, the
 * rest of the batch is dropped and counted per point).  Under DMI_POLICY_BLOCK the batch is
 * issued in as few launches as the device ring's size allows, each waiting for its room.
 * *n_done [host, optional]: how many positions of the arrays have been dealt with (captured or
 * skipped) when the call returns: n unless it fails; after DMI_ERR_AGAIN call again from there.
 * Returns DMI_OK if anything was launched, else DMI_SAMPLED_OUT or DMI_POINT_DISABLED.
 */
dmi_status_t dmi_observe_batch(dmi_ring_t *ring, uint32_t n, const uint32_t *point_ids /*[host]*/,
                               const void *const *data /*[host]*/, const dmi_tensor_t *like /*[host]*/,
                               const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                               uint64_t step_id, void *hip_stream, uint32_t *n_done /*[host]*/);
dmi_status_t dmi_observe_paged_batch(dmi_ring_t *ring, uint32_t n, const uint32_t *point_ids /*[host]*/,
                                     const void *const *bases /*[host]*/, const dmi_paged_kv_t *like /*[host]*/,
                                     const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                                     uint64_t step_id, void *hip_stream, uint32_t *n_done /*[host]*/);

/*
 * dmi_observe for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It needs no ring object and calls no allocating
 * routine: the device memory a capture needs besides its input and output (control words,
 * counters, the staged request table) is a 128 KiB array that the library's code object holds
 * on every GPU for the life of the process.
 * Runs on the calling thread's current HIP device.  Launches, on hip_stream, two one-workgroup
 * launches that reset the control words and stage the request table, then the capture kernel
 * dmi_observe would launch, and returns.  The record, byte for byte the one dmi_observe would
 * produce with sequence number `seq` and this rank_tag, is written at out[0 ..) [device,
 * 64-byte aligned]; its size is in its header (bytes 48..55) and, when the selection has no
 * keep vector, in *record_bytes [host, optional] (with one: an upper bound).  Bytes of `out`
 * behind the record are not touched.  No policy applies: nothing is sampled, dropped or waited for.
 * Limits: at most 1024 requests; the record's upper bound (dmi_record_bytes with every listed
 * row kept) must fit out_bytes (a multiple of 64): otherwise DMI_ERR_TOO_LARGE and nothing is
 * launched.  Every call on a GPU uses that GPU's one array, so calls whose kernels may overlap
 * there (different streams with no ordering between them) race; calls on one stream do not.
 * Under a stream capture, call it once outside first: the first call on a device looks the
 * array up and loads the kernels.
 */
dmi_status_t dmi_observe_into(uint32_t point_id, const dmi_tensor_t *tensor /*[host]*/,
                              const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                              uint64_t seq, uint64_t step_id, uint32_t rank_tag, void *out /*[device]*/,
                              uint64_t out_bytes, uint64_t *record_bytes /*[host]*/, void *hip_stream);

/* Move committed bytes from the device ring to the host ring (section 4.3, drain
 * stage).  Copies what is committed and fits the host ring's free space, then
 * lets the device reuse the drained span.  *bytes_moved [host, optional] = bytes
 * whose copy this call issued.  With DMI_DRAIN_FLUSH: DMI_OK means that every record of
 * every observe issued before the call has arrived in the host ring and can be polled,
 * whoever issued its copy (this call or the library's drain thread); DMI_ERR_AGAIN if
 * the host ring filled up before everything was moved (release and call again)
 * or the observes did not commit within block_timeout_ms. */
dmi_status_t dmi_drain(dmi_ring_t *ring, uint32_t flags, uint64_t *bytes_moved);

/* A whole record in the host ring: [p0, p0+n0) then, iff it straddles the end of
 * the ring, [p1, p1+n1).  Valid until released. */
typedef struct {
    const void *p0;             /* [host, pinned] */
    uint64_t n0;
    const void *p1;
    uint64_t n1;
    uint64_t seq;
} dmi_record_view_t;

/* The consumer's side of the pinned host buffer (section 4.3: the stage behind the drain takes
 * payloads out of pinned staging): up to max complete, not yet polled records, in sequence
 * order (section 4.2: ring order is hook order).  *n [host] = how many.  A record is complete
 * once the copy that carries its last byte has finished.  Views stay valid until released. */
dmi_status_t dmi_poll_host(dmi_ring_t *ring, dmi_record_view_t *out /*[host]*/, uint32_t max,
                           uint32_t *n /*[host]*/);

/* Give back the pinned space of every polled record with seq <= upto_seq_inclusive (section 4.3:
 * pinned memory is limited and is released as soon as the consumer has taken the payload; the
 * drain, and through it the backpressure policy, sees the space at once). */
dmi_status_t dmi_release_host(dmi_ring_t *ring, uint64_t upto_seq_inclusive);

/*
 * Exporter stages 2-3 (section 4.3): a library thread takes whole records out of the
 * pinned host ring, copies each into pageable memory, gives the pinned space back at once
 * (pinned memory is the scarce resource), rebuilds shape and dtype from the header and
 * slices the record by request.  While the exporter runs it is the ring's only consumer:
 * do not call dmi_poll_host / dmi_release_host yourself.  The queue of finished slices is
 * bounded by max_pageable_bytes; when it is full the exporter waits, and the pressure
 * travels back through the host ring to the device ring, where the backpressure policy
 * decides (stall or drop).
 */
typedef struct {
    uint64_t seq, step_id;
    uint32_t point_id, rank_tag;
    uint32_t req_index;         /* position of the request in the record's table */
    uint32_t req_id, tok_start, tok_step;
    uint32_t n_rows, row_elems; /* this request's rows: token tok_start + j*tok_step is row j */
    uint32_t src_dtype, out_dtype, summary_mask, flags;
    const void *rows;           /* [host, pageable] n_rows x row_elems of out_dtype; NULL if NONE */
    const float *l2, *mean, *absmax;    /* n_rows values each, NULL if not requested */
    void *owner;                /* the record copy this slice points into (library-owned) */
} dmi_slice_t;
/* n_copy_threads: pageable-copy workers (0 = 3, at most 16); results come out in ring order whatever their number. */
dmi_status_t dmi_exporter_start(dmi_ring_t *ring, uint64_t max_pageable_bytes, uint32_t n_copy_threads);
/* Next slice in (seq, request) order; waits up to timeout_ms, then DMI_ERR_AGAIN. */
dmi_status_t dmi_exporter_next(dmi_ring_t *ring, dmi_slice_t *out /*[host]*/, uint32_t timeout_ms);
/* Up to max slices that are ready now (waits up to timeout_ms for the first one); *n = how many. */
dmi_status_t dmi_exporter_next_many(dmi_ring_t *ring, dmi_slice_t *out /*[host]*/, uint32_t max,
                                    uint32_t *n /*[host]*/, uint32_t timeout_ms);
/* Release n slices at once. */
dmi_status_t dmi_exporter_release_many(dmi_ring_t *ring, const dmi_slice_t *slices /*[host]*/, uint32_t n);
/* Done with a slice; the record copy is freed when all of its slices have been released. */
dmi_status_t dmi_exporter_release(dmi_ring_t *ring, const dmi_slice_t *slice /*[host]*/);
/* Stops the thread; slices not yet handed out are discarded. */
dmi_status_t dmi_exporter_stop(dmi_ring_t *ring);

/* Backpressure policy (section 4.4), effective from the next dmi_observe. */
typedef struct {
    uint32_t mode;              /* DMI_POLICY_* */
    uint32_t sample_k;          /* >= 1 */
    uint32_t sample_phase;      /* < sample_k */
} dmi_policy_t;
dmi_status_t dmi_set_policy(dmi_ring_t *ring, const dmi_policy_t *policy /*[host]*/);

/*
 * Request-granular best effort (section 4.4, "best-effort policy" and Fig. "drop-recent"):
 * when the ring is under pressure, decide on the host, before the forward step, which
 * requests of the batch stay observed; the kernels then see the decision as a keep vector.
 *   DMI_SELECT_DROP_RECENT      the most recently admitted requests are dropped first
 *   DMI_SELECT_KEEP_BY_PATTERN  requests matching the user's predicate are kept first;
 *                               within each class the most recently admitted go first
 * dmi_policy_select is a pure host function: it orders the requests (matching ones first
 * under KEEP_BY_PATTERN, then by admit_order ascending, ties by position), and keeps the
 * longest prefix of that order whose cost, sum(rows) * bytes_per_row, fits budget_bytes.
 * keep[i] [host, n_reqs bytes] is set to 1 or 0 in the caller's request order.
 */
enum { DMI_SELECT_DROP_RECENT = 0, DMI_SELECT_KEEP_BY_PATTERN = 1 };
typedef struct {
    uint32_t req_id;
    uint32_t rows;          /* rows the request contributes per observe in the coming step */
    uint64_t admit_order;   /* smaller = admitted earlier */
    uint32_t matches;       /* KEEP_BY_PATTERN: non-zero if the predicate holds for the request */
    uint32_t reserved;
} dmi_req_info_t;
dmi_status_t dmi_policy_select(uint32_t strategy, const dmi_req_info_t *reqs /*[host]*/, uint32_t n_reqs,
                               uint64_t bytes_per_row, uint64_t budget_bytes, uint8_t *keep /*[host]*/,
                               uint32_t *n_kept /*[host, optional]*/);

/* Room the device ring is sure to have once everything launched so far has run (capacity
 * minus an upper bound of undrained bytes): the budget a policy manager works with.
 * Producer thread only. */
dmi_status_t dmi_ring_free_bytes(dmi_ring_t *ring, uint64_t *free_bytes /*[host]*/);

/* Copy a keep vector into a library-owned device buffer, ordered on hip_stream before any
 * later work of that stream.  *keep_mask_dev [device] may be passed as
 * dmi_selection_t::keep_mask_dev by observes issued on the same stream; it stays valid for
 * the next three calls of this function (an observe that passes an older address gets
 * undefined results).  The library keeps a host copy of each vector it uploaded: observes that
 * use one are admitted and accounted with the record's real size, so dmi_ring_free_bytes stays
 * meaningful under masking; for a caller-owned keep vector every listed request counts.
 * Updating the vector between steps does not change what is launched, only what the
 * launches copy (section 4.4). */
dmi_status_t dmi_set_keep_mask(dmi_ring_t *ring, const uint8_t *keep /*[host]*/, uint32_t n_reqs,
                               void *hip_stream, const uint8_t **keep_mask_dev /*[host]*/);

/*
 * Replayable steps (section 4.4, policy manager; section 4.1 on graph compatibility).
 *
 * Serving engines capture a forward step once into a graph and replay it.  A capture
 * launch issued by dmi_observe carries its sequence number, step id and policy as kernel
 * arguments, which a graph would freeze.  A dmi_step_t is a fixed list of capture launches
 * that read those values from device memory instead, so the launches can be recorded into
 * the caller's hipGraph together with the caller's own kernels:
 *
 *     dmi_step_create(ring, max_observes, &step);
 *     dmi_step_capture_begin(step);
 *       hipStreamBeginCapture(stream, ...);               // the caller's capture
 *         ... forward pass, with dmi_step_observe(step, point, tensor, sel, xf, stream, &node)
 *             where a HookPoint sits ...
 *       hipStreamEndCapture(stream, &graph);
 *     dmi_step_seal(step);
 *     per step:
 *         dmi_step_update(step, node, reqs, n_reqs);      // optional: new batch composition
 *         dmi_step_begin(step, step_id, stream);          // the policy manager's turn
 *         hipGraphLaunch(graph_exec, stream);             // exactly once per dmi_step_begin
 *         dmi_step_end(step, stream);
 *
 * What stays fixed between replays: the list of launches, their source tensors (address,
 * shape, strides), transforms, request counts, the addresses of keep vectors and row
 * indices.  What may change: the contents of source tensors, of keep_mask_dev and
 * row_index_dev vectors (caller-owned device memory, rewritten on the stream before the
 * replay; a vector from dmi_set_keep_mask rotates and is not suitable), request tables
 * (dmi_step_update), step id, backpressure policy and sampling (dmi_set_policy).  Hook
 * filtering applies when the step is captured: dmi_step_observe of a disabled point
 * returns DMI_POINT_DISABLED and adds nothing to the graph.
 *
 * Records, sequence numbers, drops and counters are the same as if the step's observes
 * had been issued by dmi_observe in the same order.  dmi_observe may be used between
 * steps (not between dmi_step_begin and dmi_step_end).  All of these are producer-thread
 * calls.  Destroy a step after its last replay has finished and before its ring.
 */
typedef struct dmi_step dmi_step_t;
#define DMI_STEP_MAX_OBSERVES 256u   /* records per step */
/* Allocates the step's device-side parameter block and request-table space (not under capture). */
dmi_status_t dmi_step_create(dmi_ring_t *ring, uint32_t max_observes, dmi_step_t **out /*[host]*/);
dmi_status_t dmi_step_destroy(dmi_step_t *step);
/* Opens the step for dmi_step_observe*.  Until dmi_step_seal the library's own threads
 * (drain thread, exporter) make no HIP call, so a capture in the global capture mode is
 * not disturbed by them; the caller's other threads must not call into this ring either. */
dmi_status_t dmi_step_capture_begin(dmi_step_t *step);
/* As dmi_observe / dmi_observe_paged without step id: validates, appends the launch to the
 * step and issues it on hip_stream, which must be capturing (DMI_ERR_INVALID_ARG otherwise).
 * Makes no HIP call besides the capture-status query and the kernel launch.
 * *node [host, optional] = index of the record in the step (what dmi_step_update takes).
 * Returns DMI_POINT_DISABLED (no launch) for a disabled point. */
dmi_status_t dmi_step_observe(dmi_step_t *step, uint32_t point_id, const dmi_tensor_t *tensor /*[host]*/,
                              const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                              void *hip_stream, uint32_t *node /*[host]*/);
dmi_status_t dmi_step_observe_paged(dmi_step_t *step, uint32_t point_id, const dmi_paged_kv_t *kv /*[host]*/,
                                    const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                                    void *hip_stream, uint32_t *node /*[host]*/);
/* As dmi_observe_batch / dmi_observe_paged_batch inside a step: the n tensors become n
 * consecutive records of the step, written by one launch (two beyond 128 tensors).
 * *node = index of the first of them.  Disabled points are left out; DMI_POINT_DISABLED if all are. */
dmi_status_t dmi_step_observe_batch(dmi_step_t *step, uint32_t n, const uint32_t *point_ids /*[host]*/,
                                    const void *const *data /*[host]*/, const dmi_tensor_t *like /*[host]*/,
                                    const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                                    void *hip_stream, uint32_t *node /*[host]*/);
dmi_status_t dmi_step_observe_paged_batch(dmi_step_t *step, uint32_t n, const uint32_t *point_ids /*[host]*/,
                                          const void *const *bases /*[host]*/, const dmi_paged_kv_t *like /*[host]*/,
                                          const dmi_selection_t *sel /*[host]*/, const dmi_transform_t *xf /*[host]*/,
                                          void *hip_stream, uint32_t *node /*[host]*/);
/* Closes the step; the library's threads resume. */
dmi_status_t dmi_step_seal(dmi_step_t *step);
/* Replace the request table of record `node` of the step (host side; it reaches the device with the
 * next dmi_step_begin).  Launches captured with an identical table share it and are
 * updated together.  n_reqs must be the captured count; rows must lie inside every
 * tensor concerned; a launch captured with one row per request and no keep vector keeps
 * that shape (and, where request i sat in row first + i, that placement), otherwise
 * DMI_ERR_INVALID_ARG: capture again. */
dmi_status_t dmi_step_update(dmi_step_t *step, uint32_t node, const dmi_req_sel_t *reqs /*[host]*/, uint32_t n_reqs);
/* Before each replay, on the stream the graph is about to be launched on: sampling
 * (returns DMI_SAMPLED_OUT: the graph is still launched, its capture kernels then do
 * nothing and take no sequence numbers), admission (DMI_POLICY_BLOCK: waits on the host,
 * as dmi_observe does, until all records of the step are sure to fit; DMI_ERR_TOO_LARGE
 * if they can never fit together; DMI_ERR_AGAIN after block_timeout_ms), upload of
 * changed tables and of the step's parameters (one small launch on hip_stream). */
dmi_status_t dmi_step_begin(dmi_step_t *step, uint64_t step_id, void *hip_stream);
/* After the graph launch, same stream: accounts for the step's launches. */
dmi_status_t dmi_step_end(dmi_step_t *step, void *hip_stream);

/* Hook filtering (section 4.4): a disabled point launches nothing. */
dmi_status_t dmi_point_enable(dmi_ring_t *ring, uint32_t point_id, int enabled);

typedef struct {
    uint64_t observed_calls, launched_records;
    uint64_t captured_records, captured_rows, captured_bytes;   /* committed on the device */
    uint64_t dropped_records, dropped_rows, dropped_bytes;      /* discarded by drop-newest */
    uint64_t sampled_out_calls, sampled_out_rows, disabled_calls;
    uint64_t drained_bytes, released_bytes, drain_batches;
    uint64_t block_wait_ns;
    uint64_t dev_ring_high_water, host_ring_high_water;
    uint64_t bad_rows;          /* rows whose row_index_dev / block-table entry left the source:
                                   stored as zeros (read from the device, synchronises the library's
                                   own stream only) */
} dmi_stats_t;
/* Counters of the observation path (section 4.4: what was dropped under best effort is counted,
 * section 6 reports overhead and volume from such counters).  Device-side counters (captured_*,
 * dropped_*) cover the launches whose completion the library has observed: after
 * dmi_drain(DMI_DRAIN_FLUSH) that is all of them.  May be called from any thread; each value is
 * read atomically, the set of values is not one consistent snapshot while other threads run. */
dmi_status_t dmi_get_stats(dmi_ring_t *ring, dmi_stats_t *out /*[host]*/);
/* Records of one observation point discarded under best effort (section 4.4: drops are made
 * visible per hook, so that a consumer knows which points have gaps).  Reads the device's
 * counter: synchronises the library's own stream only. */
dmi_status_t dmi_get_point_drops(dmi_ring_t *ring, uint32_t point_id, uint64_t *n /*[host]*/);

/* Pure host helpers (no GPU needed). */
uint64_t dmi_record_bytes(uint32_t n_reqs, uint64_t n_rows, uint32_t row_elems, uint32_t out_dtype,
                          uint32_t summary_mask);
const char *dmi_last_error(void);
const char *dmi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DMI_H */
