// Internal interface between the host runtime (dmi_host.hip) and the device code
// (dmi_kernels.hip).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dmi {

constexpr uint32_t kThreads = 256;          // 4 wavefronts of 64 lanes per workgroup
constexpr uint32_t kMaxGrid = 1u << 22;     // workgroups per tensor of one launch
constexpr uint32_t kLdsTableMax = 1024;     // request tables up to this size are cached in LDS
constexpr uint32_t kDecodeMaxListed = 1024; // most rows a ragged selection may list to take the decode-shaped kernel
constexpr uint32_t kMaxBatch = 128;         // most tensors one batched launch captures

// One slot per launch, written by workgroup 0 of the launch: where the head stands
// after it, and the running counters.  Slot seq % kCommitSlots lives in device memory;
// the host fetches it into a pinned mirror behind an event recorded after launch `seq`
// (the role of the paper's CPU-side meta ring; the kernel-end release takes the place
// of its in-kernel fence).
constexpr uint32_t kCommitSlots = 1024;
struct CommitSlot {
    uint64_t seq_plus1;
    uint64_t head;
    uint64_t captured_records, captured_rows, captured_bytes;
    uint64_t dropped_records, dropped_rows, dropped_bytes;
};

// Control block in device memory.  Offsets are logical stream offsets.
//
// Launches of one ring run one after another (stream order), so the head needs no
// atomic reservation: the n-th launch reads head[n & 1], which the previous launch
// wrote and nobody writes during this one, and its workgroup 0 writes
// head[(n + 1) & 1], which nobody reads during this one.  No workgroup has to be
// the last one, so the kernel has no completion counter and no fence.  The tail the
// drop-newest decision uses travels the same way (tail_for): one lane of a launch reads the
// drained-up-to mark from a word in pinned host memory that the drain side keeps current
// with plain CPU stores (no copy, launch or event of the drain ever enters a GPU queue
// for it) and leaves it for the next launch.
struct DevCtrl {
    uint64_t head[2];               // next free stream byte, double buffered by launch parity
    uint64_t tail_for[2];           // the tail as the previous launch saw it, same scheme
    uint64_t tail;                  // drained-up-to mark as the last replayable step's begin launch read it
    uint64_t captured_records, captured_rows, captured_bytes;
    uint64_t dropped_records, dropped_rows, dropped_bytes;
    uint64_t bad_rows;              // rows whose device-side index left the tensor (stored as zeros)
    uint32_t point_drops[4096];
    CommitSlot slots[kCommitSlots];
};

// Per-step values of a replayable step (device memory, one block per step object).
// Kernels launched as part of such a step take from here what an ordinary launch gets as
// kernel arguments, so their launches can sit in a captured graph: the graph is replayed
// unchanged and only this block (and the request tables) are rewritten between replays,
// the way the paper's keep/drop vector is (section 4.4).
struct StepParams {
    uint64_t seq_base;              // sequence number of the step's first observe
    uint64_t step_id;
    uint64_t tail_floor;            // the host's view of the tail when the step was begun
    uint32_t flags;                 // bit 0: drop-newest policy; bit 1: step sampled out, capture nothing
    uint32_t pad;
};
constexpr uint32_t kStepDropNewest = 1u, kStepSkip = 2u;

// A batched launch captures several tensors that share shape, selection and transform: one
// record each, at consecutive sequence numbers, laid down one behind the other exactly as
// consecutive single launches would.  Workgroups with blockIdx.y = i work on tensor i; what
// differs between the tensors travels in this second argument block (a single launch is a
// batch of one).
struct BatchArgs {
    const uint8_t *src[kMaxBatch];  // dense: the tensor's data; paged: the cache's base
    uint32_t point[kMaxBatch];      // observation point of each record
};

// What the general capture kernel reads (its argument block: five 64-byte lines).
struct CaptureKernelArgs {
    // source (the data pointer itself is in BatchArgs)
    int64_t row_stride_b;           // dense: bytes between rows
    int64_t n_src_rows;             // dense: rows in the tensor; paged: physical blocks
    int64_t block_stride_b, slot_stride_b, head_stride_b;
    const int32_t *block_table;
    int64_t bt_stride;
    uint32_t block_size;
    uint32_t n_seg;                 // segments per row (1, or selected heads)
    uint32_t seg_units;             // units per segment
    uint32_t heads_sel[8];
    // selection (device slab)
    const uint4 *req_table;         // {req_id, tok_start, tok_step, tok_count}
    const uint32_t *row0;           // dense: row_base + tok_start; paged: row of the block table
    const uint8_t *keep_mask;
    const int32_t *row_index;
    uint32_t n_reqs;
    uint32_t paged;
    // transform / record
    uint32_t src_dtype, out_dtype, summary_mask, rec_flags;
    uint32_t row_elems;
    uint32_t units_per_row;
    uint32_t rows_per_wg;           // summary kernels: 1 (a workgroup per row) or 4 (a wavefront per row)
    uint32_t n_batch, rank_tag;     // n_batch = gridDim.y
    uint64_t seq, step_id;          // seq: of the launch's first record
    // ring
    uint8_t *ring;
    uint64_t cap;
    DevCtrl *ctrl;
    CommitSlot *cslot;              // this launch's commit slot (device memory)
    uint64_t tail_floor;            // the host's view of the tail when the launch was issued
    const uint64_t *tail_src;       // pinned host word holding the drained-up-to mark (NULL: not read)
    uint32_t simple;                // no keep mask and every request contributes exactly one row
    uint32_t upr_shift;             // log2(units_per_row) if that is a power of two, else 32
    uint32_t bs_shift, seg_shift;   // same for block_size and seg_units
    uint32_t drop_newest;
    uint32_t force_drop;            // every record of this launch is dropped (the host knows none can fit)
    uint32_t n_tail_drop;           // records of the caller's list behind the n_batch launched ones that the host
                                    // knows cannot fit: this launch only counts them (BatchArgs::point has their
                                    // points behind the launched ones'); they take the sequence numbers that follow
    uint32_t table_in_lds;
    // launch chain: which copy of head / tail_for this launch reads (it writes the other)
    uint32_t par_in;
    // replayable steps: seq = step->seq_base + node, step id, tail floor and policy from *step
    uint32_t node;
    const StepParams *step;
};

// The host's plan of one launch: the kernel's arguments plus what only the launchers need
// (the decode-shaped kernel gets its own, smaller block made from this).
struct CaptureArgs : CaptureKernelArgs {
    const uint8_t *src;             // the tensor (the first one of a batch); goes into BatchArgs::src
    uint32_t point_id;              // same, BatchArgs::point
    uint32_t one_row_each;          // every request lists exactly one row (a keep vector may still drop some)
    uint32_t listed_rows;           // rows the selection lists (all requests kept)
    const uint32_t *row_map;        // decode-shaped kernel, requests listing several rows: source row of every
                                    // output row, written by the host behind the request table
    uint32_t lds_bytes;
    // record geometry and header words, filled by the host when it knows them exactly (no keep
    // mask: the row count is the listed one); used by the decode-shaped kernel
    uint32_t hdr[16];
    uint64_t off_payload, off_sum, sum_arr, record_bytes, payload_bytes;
    uint32_t rows_consecutive;      // request i's row is row_first + i: no table lookup needed
    uint32_t row_first;
};

// Launchers (dmi_kernels.hip).  All return the launch's hipError_t.
hipError_t launch_capture(const CaptureArgs &a, const BatchArgs &b, uint32_t grid, bool vec16, hipStream_t s);
// decode-shaped captures: bf16 source (fp16 if stored as it is), dense, one row per request (with or without a keep
// vector; with one, at most 1024 requests), 16-byte movable rows of at most 1024 units;
// grid is n_reqs + 1
bool decode_kernel_applies(const CaptureArgs &a, bool vec16);
hipError_t launch_capture_decode(const CaptureArgs &a, const BatchArgs &b, hipStream_t s);
hipError_t launch_upload(uint32_t *dst, const uint32_t *words, uint32_t n_words, hipStream_t s);
// start of a replayable step: writes *step and, if par_from != par_to, carries head and
// tail_for over to the copy the step's first launch reads
hipError_t launch_step_begin(DevCtrl *ctrl, StepParams *step, StepParams v, uint32_t par_from, uint32_t par_to,
                             const uint64_t *host_tail, hipStream_t s);
// zeroes head / tail copies and the running counters of a control block
hipError_t launch_ctrl_reset(DevCtrl *ctrl, hipStream_t s);
hipError_t launch_fetch_slot(const CommitSlot *src, CommitSlot *dst_host, hipStream_t s);
hipError_t launch_drain_kernel(const uint8_t *ring, uint64_t cap, uint8_t *host_ring, uint64_t host_cap,
                               uint64_t from, uint64_t nbytes, uint32_t grid, hipStream_t s);
uint32_t capture_lds_bytes(uint32_t n_reqs, bool index_mode, bool table_in_lds);

}  // namespace dmi
