// Host-side internals shared by the runtime's source files (dmi_host.hip: rings, admission,
// commit discovery, drain, C ABI core; dmi_step.hip: replayable steps; dmi_exporter.hip:
// exporter stages 2-3).  Not part of the public ABI.
#pragma once
#include "dmi.h"
#include "dmi_debug.h"
#include "dmi_internal.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

namespace dmi {
namespace host {

// Records the message for dmi_last_error() (thread-local) and returns `code`.
dmi_status_t fail(dmi_status_t code, const char *fmt, ...);

#define HIP_TRY(expr)                                                                     \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess)                                                             \
            return ::dmi::host::fail(DMI_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline uint64_t now_ns()
{
    return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
               std::chrono::steady_clock::now().time_since_epoch()).count();
}

inline uint64_t pad64(uint64_t n) { return (n + 63u) & ~63ull; }

inline uint32_t dtype_size(uint32_t dt)
{
    switch (dt) {
    case DMI_DTYPE_BF16: case DMI_DTYPE_FP16: return 2;
    case DMI_DTYPE_FP32: return 4;
    case DMI_DTYPE_FP8_E4M3FN: return 1;
    default: return 0;
    }
}

inline bool transform_ok(uint32_t src, uint32_t out)
{
    if (src != DMI_DTYPE_BF16 && src != DMI_DTYPE_FP16 && src != DMI_DTYPE_FP32) return false;
    if (out == DMI_DTYPE_NONE || out == src) return true;
    return src == DMI_DTYPE_BF16 && (out == DMI_DTYPE_FP16 || out == DMI_DTYPE_FP8_E4M3FN);
}

constexpr uint32_t kSlabSlots = 64;
constexpr uint32_t kSelCache = 4;

struct SelCache {
    bool valid = false;
    bool paged = false;
    hipStream_t stream = nullptr;
    uint32_t slot = 0;
    std::vector<uint32_t> words;
};


// One record copied out of the pinned ring (exporter stage 2) and shared by its slices.
struct RecordCopy {
    uint8_t *bytes;
    uint64_t size;              // the record's bytes
    uint64_t cap;               // the buffer's bytes (>= size: buffers are reused, see PoolBuf)
    std::atomic<uint32_t> refs;
};

// An idle pageable buffer of the exporter, kept for the next record of about this size.
struct PoolBuf {
    uint8_t *p;
    uint64_t cap;
};

struct ExportJob {
    dmi_record_view_t view;
    uint64_t ticket;
};

struct ExportDone {
    uint64_t seq;
    RecordCopy *rc;
    std::vector<dmi_slice_t> slices;
};

struct Geometry {
    uint32_t src_dtype, row_elems, n_seg, seg_elems;
    bool vec16;
};

// What a capture launch is, apart from when it runs and where its table lives.
struct Plan {
    uint64_t listed = 0;        // rows the selection lists
    uint64_t ub = 0;            // record bytes if every request is kept (or exactly, see size_known)
    uint64_t rows_known = 0;    // rows of the record when size_known
    bool size_known = false;    // no keep vector, or one the host has a copy of: ub is the record's size
    uint32_t grid = 1;
    bool decode = false;        // the decode-shaped kernel applies
    bool row_map = false;       // ... and wants the source row of every listed row behind the table
};

// Where a planned launch writes and what it stamps into its header.  `masks`, when given, is the
// ring whose dmi_set_keep_mask buffers the plan may recognise (the host knows their contents).
struct PlanEnv {
    uint8_t *ring;
    uint64_t cap;
    uint64_t host_cap;      // 0: the records do not travel on to a host ring
    DevCtrl *ctrl;
    uint32_t rank_tag;
    const dmi_ring *masks;
};

// What the launches between two probes add when the host can tell without asking the
// device: records whose size the host knows (no keep vector, or one it has a copy of), under
// the completeness policy, where none is dropped, or under best effort while the host knows
// where the head stands and decides itself which records fit.
struct Delta {
    uint64_t bytes = 0, records = 0, rows = 0;              // captured
    uint64_t drop_bytes = 0, drop_records = 0, drop_rows = 0;   // dropped, by the host's own decision
};

struct Probe {
    hipEvent_t ev;          // recorded on the producer's stream behind the launches (and the slot fetch)
    uint64_t covers;        // every launch with seq < covers was enqueued before ev
    uint64_t launches;      // how many capture launches that is
    bool fetched;           // the commit slot of launch covers-1 was copied to the host mirror
    Delta delta;            // else: what the launches since the previous probe added
};

}  // namespace host
}  // namespace dmi

using namespace dmi;         // internal header: the structs below are made of these types
using namespace dmi::host;

struct dmi_ring {
    dmi_ring_config_t cfg{};
    int dev = 0;
    uint8_t *dev_ring = nullptr;
    uint64_t dev_cap = 0;
    uint8_t *host_ring = nullptr, *host_ring_dev = nullptr;
    uint64_t host_cap = 0;
    DevCtrl *dctrl = nullptr;
    CommitSlot *hslots = nullptr, *hslots_dev = nullptr;   // pinned mirror of DevCtrl::slots
    hipStream_t ctl_stream = nullptr;                      // statistics reads, set-up launches
    uint8_t *mask_buf = nullptr;                           // 4 rotating keep vectors of max_reqs bytes
    uint32_t mask_rr = 0, mask_stride = 0;
    std::vector<uint8_t> mask_host[4];                     // what dmi_set_keep_mask last put into each of them
    uint32_t *slab = nullptr;
    uint32_t slab_slot_words = 0, next_slab = 0, max_reqs = 0;
    SelCache cache[kSelCache];
    std::vector<uint32_t> sel_scratch;
    uint32_t cache_rr = 0;
    hipStream_t drain_stream = nullptr;
    uint32_t block_timeout_ms = 2000;

    // policy (set by the producer thread or between steps)
    std::atomic<uint32_t> mode{DMI_POLICY_BLOCK}, sample_k{1}, sample_phase{0};
    std::vector<uint8_t> point_off;

    // producer side
    std::atomic<uint64_t> next_seq{0};                     // launches issued so far
    std::atomic<void *> last_stream{nullptr};
    std::atomic<uint64_t> last_launch_ns{0};
    std::deque<std::pair<uint64_t, uint64_t>> inflight;    // (seq, upper bound of record bytes)
    uint64_t inflight_sum = 0;
    uint64_t unprobed_launches = 0, unprobed_bytes = 0, probe_bytes = 8u << 20;
    uint32_t chain_par = 0;                                // which copy of head / tail_for the next launch reads
    std::atomic<uint64_t> launches{0};                     // capture launches issued so far
    std::atomic<uint64_t> confirmed_launches{0};           // ... and how many of them are known to have finished
    // Does the host know where the device head will stand once everything launched so far has run?
    // It does while every launch since the last confirmed state had an outcome the host could tell
    // in advance; it then decides best-effort drops itself instead of leaving them to the kernel,
    // provided it is not running far ahead of the GPU (the drained mark it would decide on ages
    // while the launch waits in the queue; the kernel decides on a fresher one).
    bool head_exact = true;
    uint64_t exact_head = 0;
    bool step_open = false;                                // between dmi_step_begin and dmi_step_end
    std::atomic<int> quiet{0};                             // a capture is open: library threads make no HIP call
    std::atomic<bool> bg_parked{false};

    // commit discovery: events recorded behind launches ("probes"), queried in order
    std::mutex pmu;
    std::deque<Probe> probes;
    std::vector<hipEvent_t> probe_pool;
    Delta window;                                          // launches since the last probe (under pmu)
    bool window_exact = true;
    uint64_t probed_upto = 0;                              // launches with seq < this have a probe behind them
    std::atomic<uint64_t> confirmed{0};                    // launches with seq < this have finished
    std::atomic<uint64_t> committed{0};                    // device head after launch confirmed-1
    uint64_t snap[6] = {0, 0, 0, 0, 0, 0};                 // counters of the last confirmed slot

    // drain / host ring state
    std::mutex mu;
    uint64_t drain_issued = 0;
    uint64_t drain_issued_records = 0;                     // captured records below drain_issued (a lower bound
                                                           // while a batch stops short of the committed head)
    std::atomic<uint64_t> drain_done{0};
    // The drain stream carries the batch copies only (no launch, no event, no small copy: any
    // of these is a packet on a second compute queue that waits for the copy in front of it, and
    // a waiting packet there slows every dispatch of the producer's queue by a microsecond or so).  A batch is known to be
    // done when the whole stream is idle; the drained-up-to mark reaches the kernels through a
    // pinned host word that they read themselves.
    volatile uint64_t *htail = nullptr;                    // pinned, coherent
    const uint64_t *htail_dev = nullptr;                   // its device address
    uint64_t poll_cursor = 0, released = 0;
    std::deque<std::pair<uint64_t, uint64_t>> polled;      // (seq, end offset)

    // statistics kept on the host
    std::atomic<uint64_t> observed_calls{0}, sampled_out_calls{0}, sampled_out_rows{0}, disabled_calls{0},
        drained_bytes{0}, released_bytes{0}, drain_batches{0}, block_wait_ns{0}, dev_high{0}, host_high{0};

    std::thread bg;
    std::atomic<bool> stop{false};

    // exporter stages 2-3
    std::thread exporter;
    std::atomic<bool> exp_stop{false}, exp_running{false};
    std::mutex emu;
    std::condition_variable ecv_data, ecv_space;
    std::deque<dmi_slice_t> slices;
    uint64_t exp_bytes = 0, exp_max_bytes = 0, next_emit = 0;
    std::vector<std::thread> exp_workers;
    std::mutex jmu;
    std::condition_variable jcv;
    std::deque<ExportJob> jobs;
    std::map<uint64_t, ExportDone> done_jobs;
    std::atomic<uint64_t> exp_records{0}, exp_copied_bytes{0};
    std::mutex pool_mu;                     // guards exp_pool and exp_pool_bytes; taken after emu, never before it
    std::vector<PoolBuf> exp_pool;          // idle buffers, oldest first
    uint64_t exp_pool_bytes = 0;
    std::atomic<uint64_t> exp_mallocs{0}, exp_reuses{0};
};

// A replayable step (section 4.4, policy manager): a fixed list of capture launches that
// take sequence base, step id, tail floor and policy from device memory.
struct StepTable {                  // one request table, shared by the nodes captured with the same selection
    std::vector<uint32_t> words;    // as selection_words() lays them out
    std::vector<dmi_req_sel_t> reqs;
    bool paged = false;
    bool row_map = false;           // carries the source row of every listed row behind the table
    bool dirty = true;              // staged on the host, not yet on the device
    uint32_t slot = 0;
};

struct StepNode {                   // one launch of the step: n_batch records from first_rec on
    CaptureArgs a;
    uint32_t first_rec = 0, n_batch = 1;
    Plan pl;                        // per record
    Geometry geo;
    dmi_transform_t xf;
    uint32_t point_id = 0;
    uint32_t table = 0;
    bool index_mode = false, masked = false;
    uint32_t n_seqs = 0;            // paged: rows of the block table
};

struct dmi_step {
    dmi_ring *r = nullptr;
    uint32_t max_nodes = 0;
    std::vector<StepNode> nodes;
    std::vector<uint32_t> rec_launch;   // record of the step -> the launch that writes it
    std::vector<StepTable> tables;
    StepParams *dparams = nullptr;  // device
    uint32_t *slab = nullptr;       // device: max_nodes table slots
    bool open = false, sealed = false, begun = false, skipped = false, drop_newest = false;
    uint64_t sum_ub = 0, sum_listed = 0, seq_base = 0;
};

namespace dmi {
namespace host {

// dmi_host.hip
dmi_status_t record_probe(dmi_ring *r);
dmi_status_t advance_commits(dmi_ring *r, bool block);
uint64_t head_upper_bound(dmi_ring *r);
dmi_status_t wait_for_room(dmi_ring *r, uint64_t ub);
dmi_status_t drain(dmi_ring *r, bool wait, uint64_t *moved, bool *host_full = nullptr);
dmi_status_t commit_slot_room(dmi_ring *r, uint32_t n);
void selection_words(const dmi_req_sel_t *reqs, uint32_t n, bool paged, bool row_map, std::vector<uint32_t> &words);
PlanEnv plan_env(const dmi_ring *r);
uint32_t plan_grid(const CaptureArgs &a, uint32_t nb);
bool batch_takes_decode_kernel(const CaptureArgs &a, uint32_t nb);
dmi_status_t check_batch_sources(uint32_t n, const void *const *data, uint32_t es, bool *all16);
dmi_status_t plan_capture(const PlanEnv &env, uint32_t point_id, const dmi_selection_t *sel, const dmi_transform_t *xf,
                          const Geometry &geo, CaptureArgs &a, Plan &pl, bool fixed_row_count_ok);
dmi_status_t check_dense_rows(const dmi_req_sel_t *reqs, uint32_t n, int64_t T);
dmi_status_t check_paged_rows(const dmi_req_sel_t *reqs, uint32_t n, uint32_t n_seqs, uint32_t block_size,
                              int64_t bt_stride);
dmi_status_t prep_dense(const dmi_tensor_t *t, const dmi_selection_t *sel, Geometry &geo, CaptureArgs &a);
dmi_status_t prep_paged(const dmi_paged_kv_t *kv, const dmi_selection_t *sel, Geometry &geo, CaptureArgs &a);
dmi_status_t poll_host_impl(dmi_ring *r, dmi_record_view_t *out, uint32_t max, uint32_t *n);
dmi_status_t release_host_impl(dmi_ring *r, uint64_t upto);

}  // namespace host
}  // namespace dmi
