// Host runtime of the capture-and-stage library: ring ownership, policy gate and
// admission (paper section 4.4), kernel launches for dmi_observe (section 4.2), the
// drain stage and pinned host ring (section 4.3), and the core of the C ABI of include/dmi.h
// (replayable steps: dmi_step.hip; exporter: dmi_exporter.hip).
#include "dmi_ring.h"

using namespace dmi;
using namespace dmi::host;

namespace dmi {
namespace host {

static thread_local std::string g_err;

dmi_status_t fail(dmi_status_t code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

const char *last_error_cstr() { return g_err.c_str(); }

}  // namespace host
}  // namespace dmi

namespace dmi {
namespace host {

void atomic_max(std::atomic<uint64_t> &a, uint64_t v)
{
    uint64_t cur = a.load(std::memory_order_relaxed);
    while (cur < v && !a.compare_exchange_weak(cur, v, std::memory_order_relaxed)) {}
}

// Record an event behind everything launched so far (no-op if that is already covered).
// If the host cannot tell what those launches added (drop-newest, keep vectors), the
// newest launch's commit slot is fetched into the pinned mirror in front of the event.
// Both go onto the producer's own stream: a launch on a second hardware queue that waits
// for an event of this one slows every dispatch here by a microsecond or so while it
// waits, far more than a small launch every sixteenth capture costs in line.
dmi_status_t record_probe(dmi_ring *r)
{
    std::lock_guard<std::mutex> lk(r->pmu);
    const uint64_t launched = r->next_seq.load(std::memory_order_acquire);
    if (launched <= r->probed_upto) return DMI_OK;
    hipEvent_t ev;
    if (r->probe_pool.empty()) HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    else { ev = r->probe_pool.back(); r->probe_pool.pop_back(); }
    hipStream_t us = (hipStream_t)r->last_stream.load(std::memory_order_acquire);
    const bool fetch = !r->window_exact;
    if (fetch) {
        const uint32_t slot = (uint32_t)((launched - 1u) % kCommitSlots);
        HIP_TRY(launch_fetch_slot(&r->dctrl->slots[slot], r->hslots_dev + slot, us));
    }
    HIP_TRY(hipEventRecord(ev, us));
    r->probes.push_back({ev, launched, r->launches.load(std::memory_order_relaxed), fetch, r->window});
    r->window = Delta();
    r->window_exact = true;
    r->probed_upto = launched;
    return DMI_OK;
}

// Take note of finished probes: the slot of the newest launch they cover says where the
// device head stands.  With block=true waits for the oldest outstanding probe.
dmi_status_t advance_commits(dmi_ring *r, bool block)
{
    std::lock_guard<std::mutex> lk(r->pmu);
    while (!r->probes.empty()) {
        Probe &p = r->probes.front();
        hipError_t e = block ? hipEventSynchronize(p.ev) : hipEventQuery(p.ev);
        block = false;
        if (e == hipErrorNotReady) break;
        if (e != hipSuccess) return fail(DMI_ERR_HIP, "commit event: %s", hipGetErrorString(e));
        if (p.fetched) {
            const volatile CommitSlot &sl = r->hslots[(p.covers - 1u) % kCommitSlots];
            std::atomic_thread_fence(std::memory_order_acquire);
            if (sl.seq_plus1 != p.covers)
                return fail(DMI_ERR_CLOSED, "commit slot of launch %llu holds %llu",
                            (unsigned long long)(p.covers - 1u), (unsigned long long)sl.seq_plus1);
            r->snap[0] = sl.captured_records; r->snap[1] = sl.captured_rows; r->snap[2] = sl.captured_bytes;
            r->snap[3] = sl.dropped_records;  r->snap[4] = sl.dropped_rows;  r->snap[5] = sl.dropped_bytes;
            r->committed.store(sl.head, std::memory_order_release);
        } else {
            // state after the previous probe is exact, and so is what came since
            r->snap[0] += p.delta.records; r->snap[1] += p.delta.rows; r->snap[2] += p.delta.bytes;
            r->snap[3] += p.delta.drop_records; r->snap[4] += p.delta.drop_rows; r->snap[5] += p.delta.drop_bytes;
            r->committed.store(r->committed.load(std::memory_order_relaxed) + p.delta.bytes,
                               std::memory_order_release);
        }
        r->confirmed.store(p.covers, std::memory_order_release);
        r->confirmed_launches.store(p.launches, std::memory_order_release);
        r->probe_pool.push_back(p.ev);
        r->probes.pop_front();
    }
    return DMI_OK;
}

uint64_t read_committed(const dmi_ring *r) { return r->committed.load(std::memory_order_acquire); }

// The drained-up-to mark, where the kernels read it: one pinned word, written here and read by a
// lane of a running kernel across the host link at any time, so the store is an atomic one.
static void publish_tail(dmi_ring *r, uint64_t mark)
{
    __atomic_store_n(const_cast<uint64_t *>(r->htail), mark, __ATOMIC_RELEASE);
}

// Retire finished copies (all of them at once: the drain stream is idle).  Caller holds r->mu.
dmi_status_t reap(dmi_ring *r, bool wait)
{
    if (r->drain_done.load(std::memory_order_relaxed) == r->drain_issued) return DMI_OK;
    hipError_t e = wait ? hipStreamSynchronize(r->drain_stream) : hipStreamQuery(r->drain_stream);
    if (e == hipErrorNotReady) return DMI_OK;
    if (e != hipSuccess) return fail(DMI_ERR_HIP, "drain stream: %s", hipGetErrorString(e));
    r->drain_done.store(r->drain_issued, std::memory_order_release);
    publish_tail(r, r->drain_issued);
    return DMI_OK;
}

// Issue copies for what is committed and fits the host ring.  Caller holds r->mu.
dmi_status_t drain_issue_locked(dmi_ring *r, uint64_t *moved, bool *host_full)
{
    if (moved) *moved = 0;
    if (host_full) *host_full = false;
    dmi_status_t st = reap(r, false);
    if (st != DMI_OK) return st;
    uint64_t committed, committed_records;
    {   // the head and the record count that belong to it
        std::lock_guard<std::mutex> pk(r->pmu);
        committed = read_committed(r);
        committed_records = r->snap[0];
    }
    atomic_max(r->dev_high, committed - r->drain_done.load(std::memory_order_relaxed));
    const uint64_t avail = committed - r->drain_issued;
    const uint64_t host_free = r->host_cap - (r->drain_issued - r->released);
    uint64_t n = avail < host_free ? avail : host_free;
    if (host_full) *host_full = avail > 0 && host_free == 0;
    // bounded batches: the device tail (what drop-newest decides on) moves once per batch
    const uint64_t batch = (r->dev_cap / 8u > (64u << 20) ? r->dev_cap / 8u : (64u << 20)) & ~63ull;
    if (n > batch) n = batch;
    if (n > 0) {
        const uint64_t from = r->drain_issued;
        if (r->cfg.flags & DMI_DRAIN_KERNEL) {
            uint64_t units = n / 16u;
            uint32_t grid = (uint32_t)((units + kThreads - 1) / kThreads);
            if (grid > 128u) grid = 128u;
            HIP_TRY(launch_drain_kernel(r->dev_ring, r->dev_cap, r->host_ring_dev, r->host_cap, from, n, grid,
                                        r->drain_stream));
        } else {
            uint64_t off = from, left = n;
            while (left) {
                const uint64_t s = off % r->dev_cap, d = off % r->host_cap;
                uint64_t len = left;
                if (len > r->dev_cap - s) len = r->dev_cap - s;
                if (len > r->host_cap - d) len = r->host_cap - d;
                HIP_TRY(hipMemcpyAsync(r->host_ring + d, r->dev_ring + s, len, hipMemcpyDeviceToHost,
                                       r->drain_stream));
                off += len;
                left -= len;
            }
        }
        r->drain_issued = from + n;
        if (r->drain_issued == committed) r->drain_issued_records = committed_records;
        r->drained_bytes += n;
        r->drain_batches += 1;
        atomic_max(r->host_high, r->drain_issued - r->released);
        if (moved) *moved = n;
    }
    return DMI_OK;
}

// Issue the copies and, if asked, wait for them.  The ring's lock is held only while the
// bookkeeping is touched, never across the wait: the consumer polls and releases, and the
// producer asks for room, while a copy is in flight.
dmi_status_t drain(dmi_ring *r, bool wait, uint64_t *moved, bool *host_full)
{
    uint64_t mark;
    {
        std::lock_guard<std::mutex> lk(r->mu);
        dmi_status_t st = drain_issue_locked(r, moved, host_full);
        if (st != DMI_OK) return st;
        mark = r->drain_issued;
        if (!wait || r->drain_done.load(std::memory_order_relaxed) == mark) return DMI_OK;
    }
    // everything issued up to `mark` was on the stream before this call
    hipError_t e = hipStreamSynchronize(r->drain_stream);
    if (e != hipSuccess) return fail(DMI_ERR_HIP, "drain stream: %s", hipGetErrorString(e));
    std::lock_guard<std::mutex> lk(r->mu);
    if (r->drain_done.load(std::memory_order_relaxed) < mark) {
        r->drain_done.store(mark, std::memory_order_release);
        publish_tail(r, mark);  // the span may be reused only now that its copies have run
    }
    return DMI_OK;
}

// Pop launches known to have finished; returns an upper bound of the device head once
// everything launched so far has run.  Producer thread only.
uint64_t head_upper_bound(dmi_ring *r)
{
    const uint64_t done = r->confirmed.load(std::memory_order_acquire);
    const uint64_t committed = r->committed.load(std::memory_order_acquire);
    while (!r->inflight.empty() && r->inflight.front().first < done) {
        r->inflight_sum -= r->inflight.front().second;
        r->inflight.pop_front();
    }
    return committed + r->inflight_sum;
}

// Completeness policy: wait on the host until a record of `ub` bytes is sure to fit
// (the paper's flush before the forward step, section 4.4).  Never a device-side wait.
dmi_status_t wait_for_room(dmi_ring *r, uint64_t ub)
{
    uint64_t t0 = 0;
    dmi_status_t st;
    for (;;) {
        // what the drain side has confirmed so far is enough to decide in the common case
        // (an older view only makes the bound more cautious)
        uint64_t head_ub = head_upper_bound(r);
        uint64_t tail = r->drain_done.load(std::memory_order_acquire);
        if (head_ub - tail + ub <= r->dev_cap) break;
        if ((st = advance_commits(r, false)) != DMI_OK) return st;
        head_ub = head_upper_bound(r);
        tail = r->drain_done.load(std::memory_order_acquire);
        if (head_ub - tail + ub <= r->dev_cap) break;
        if (!t0) t0 = now_ns();
        uint64_t moved = 0;
        if ((st = drain(r, true, &moved)) != DMI_OK) return st;
        if (moved) continue;
        st = record_probe(r);       // make sure the launches we wait for will report
        if (st != DMI_OK) return st;
        if (now_ns() - t0 > (uint64_t)r->block_timeout_ms * 1000000ull) {
            r->block_wait_ns += now_ns() - t0;
            return fail(DMI_ERR_AGAIN, "no room in the device ring after %u ms (host ring full or "
                                       "observes not finishing)", r->block_timeout_ms);
        }
        std::this_thread::sleep_for(std::chrono::microseconds(10));
    }
    if (t0) r->block_wait_ns += now_ns() - t0;
    return DMI_OK;
}

// A launch's commit slot is reused kCommitSlots launches later: keep fewer than that
// unconfirmed before issuing `n` more.
dmi_status_t commit_slot_room(dmi_ring *r, uint32_t n)
{
    while (r->next_seq.load(std::memory_order_relaxed) + n - r->confirmed.load(std::memory_order_acquire) >=
           kCommitSlots) {
        dmi_status_t st = record_probe(r);
        if (st == DMI_OK) st = advance_commits(r, true);
        if (st != DMI_OK) return st;
    }
    return DMI_OK;
}

// Request table as the kernels read it: n x {req_id, tok_start, tok_step, tok_count}, then
// n x first source row of the request (dense; callers have checked that it fits 32 bits)
// or its row of the block table (paged); with row_map, then the source row of every listed
// row in output order (for the decode-shaped kernel when requests list several rows).
void selection_words(const dmi_req_sel_t *reqs, uint32_t n, bool paged, bool row_map, std::vector<uint32_t> &words)
{
    words.resize((size_t)n * 5u);
    for (uint32_t i = 0; i < n; i++) {
        const dmi_req_sel_t &q = reqs[i];
        words[4u * i + 0] = q.req_id;
        words[4u * i + 1] = q.tok_start;
        words[4u * i + 2] = q.tok_step;
        words[4u * i + 3] = q.tok_count;
        words[4u * n + i] = paged ? q.row_base : q.row_base + q.tok_start;
    }
    if (row_map)
        for (uint32_t i = 0; i < n; i++)
            for (uint32_t j = 0; j < reqs[i].tok_count; j++)
                words.push_back(reqs[i].row_base + reqs[i].tok_start + j * reqs[i].tok_step);
}

// Put the request table where the kernel can read it from L2: a slab of slots in
// device memory, refilled only when the selection differs from recent ones (all
// hook points of a step share their selection).
dmi_status_t stage_selection(dmi_ring *r, const dmi_selection_t *sel, bool paged, bool row_map, hipStream_t s,
                             uint32_t *slot_out)
{
    std::vector<uint32_t> &words = r->sel_scratch;
    selection_words(sel->reqs, sel->n_reqs, paged, row_map, words);
    for (auto &c : r->cache) {
        if (!c.valid || c.stream != s || c.paged != paged || c.words.size() != words.size()) continue;
        if (words.empty() || memcmp(c.words.data(), words.data(), words.size() * 4u) == 0) {
            *slot_out = c.slot;
            return DMI_OK;
        }
    }
    const uint32_t slot = r->next_slab++ % kSlabSlots;
    for (auto &c : r->cache) if (c.valid && c.slot == slot) c.valid = false;
    if (!words.empty())
        HIP_TRY(launch_upload(r->slab + (size_t)slot * r->slab_slot_words, words.data(), (uint32_t)words.size(), s));
    SelCache &c = r->cache[r->cache_rr++ % kSelCache];
    c.valid = true; c.paged = paged; c.stream = s; c.slot = slot; c.words = words;
    *slot_out = slot;
    return DMI_OK;
}

// Fill every kernel argument that depends only on the tensor, the selection's shape and the
// transform.  Left to the caller: request table location, sequence number, step id, commit
// slot, tail floor, policy, chain parity.
// Workgroups per tensor (gridDim.x) of the general kernel for a launch of `nb` tensors.
// Work items per launch path, and a grid that gives every workgroup the same number of them:
// with a fixed grid of "as many as fit" the last round is run by a fraction of the
// workgroups while the rest idle (up to half the launch for 1 < items/grid < 2).
// kResident is what stays resident at the register budget of the widest variants.  In a batch
// (gridDim.y = nb) each workgroup stays with one tensor.
uint32_t plan_grid(const CaptureArgs &a, uint32_t nb)
{
    constexpr uint64_t kResident = 5u * 256u;
    const uint64_t listed = a.listed_rows, upr = a.units_per_row;
    // Decode-like selections (one row per request, no keep vector, dense) need no scan and no
    // search, and a workgroup's first item is loaded along with its control words: a workgroup
    // per item, each gone after one round trip, keeps more loads in flight than the resident
    // few looping over many items.
    const bool flat = a.simple && !a.paged;
    // A launch of several tensors works through them one after the other (the y index of a workgroup
    // is the slow one), and does best with short-lived workgroups of about four items each: the
    // hardware then hands out the work as workgroups retire, which evens out how unequally the
    // workgroups are served (the five that share a compute unit oldest first: with equal shares the
    // youngest ends 1.4 times as late as the oldest; and compute units differ by +-8 %), while
    // workgroups that stay for a whole tensor all have to end before the next tensor's can start,
    // and a resident set shared among the tensors leaves every tensor's tail to a few workgroups
    // (measured, 8 tensors of 10.2 k rows x 4096 bf16 -> fp8: 0.65 of the HBM peak with four items
    // per workgroup, 0.62 with two or eight, 0.59 with the resident set shared; two tensors of
    // 10.2 k x 14336: 0.65 against 0.60 and 0.59).
    constexpr uint64_t kItemsPerGroupInBatch = 4u;
    auto balanced = [nb, flat](uint64_t items) -> uint64_t {
        if (flat || items * nb <= kResident) return items;
        uint64_t rounds = (items * nb + kResident - 1u) / kResident;
        if (nb > 1u && rounds > kItemsPerGroupInBatch) rounds = kItemsPerGroupInBatch;
        return (items + rounds - 1u) / rounds;
    };
    uint64_t groups;
    if (a.summary_mask) {
        groups = balanced((listed + a.rows_per_wg - 1u) / a.rows_per_wg);
    } else if (upr >= kThreads && upr < 4u * kThreads && (4u * kThreads) % upr == 0) {
        groups = balanced((listed + 4u * kThreads / upr - 1u) / (4u * kThreads / upr));      // 2 or 4 rows per work item
    } else if (upr >= kThreads) {
        // a row's last item is shorter than its others: a grid size that shares a factor with the
        // items per row would give some workgroups only long items and others only short ones
        const uint64_t cpr = (upr + 4u * kThreads - 1u) / (4u * kThreads);
        groups = balanced(listed * cpr);
        auto gcd = [](uint64_t x, uint64_t y) { while (y) { const uint64_t t = x % y; x = y; y = t; } return x; };
        while (!flat && groups > 1u && gcd(groups, cpr) != 1u) groups++;
    } else {
        // short rows: slices of 256 units; a workgroup takes 4 per round once there are enough
        const uint64_t slices = (listed * upr + kThreads - 1u) / kThreads;
        groups = slices * nb <= kResident ? slices : balanced((slices + 3u) / 4u);
    }
    return groups < 1u ? 1u : groups > kMaxGrid ? kMaxGrid : (uint32_t)groups;
}

} }  // namespace dmi::host
namespace dmi {
// Which launches the decode-shaped kernel can take (see capture_decode_kernel).
bool decode_kernel_applies(const CaptureArgs &a, bool vec16)
{
    // one row per request (with a keep vector: up to 1024 requests), or, without a keep vector, any
    // selection of at most 1024 rows (the host then lists the source row of every output row)
    const bool shape = a.simple || (a.one_row_each && a.keep_mask && a.n_reqs <= 1024u) ||
                       (!a.keep_mask && a.listed_rows >= 1u && a.listed_rows <= kDecodeMaxListed);
    // 16-bit sources: bf16 with any supported output, fp16 as it is (or summaries only)
    const bool types = a.src_dtype == 1u || (a.src_dtype == 2u && (a.out_dtype == 2u || a.out_dtype == 0u));
    return shape && !a.paged && vec16 && types && a.units_per_row <= 4u * kThreads && a.n_reqs >= 1u;
}
}  // namespace dmi
namespace dmi { namespace host {

// Which kernel a launch of `nb` decode-shaped tensors takes.  The decode-shaped kernel is the
// quickest way through a small launch, where every dependent trip to memory counts; from
// some eight thousand rows on the general kernel's one-item workgroups are as quick or quicker
// (measured on 256 x 8192 bf16 tensors: 13.3 against 15.2 us for 8 tensors, 44 us either way for
// 32, 116 against 113 us for 80).  The caller has set a.drop_newest and a.step.
bool batch_takes_decode_kernel(const CaptureArgs &a, uint32_t nb)
{
    if (nb == 1u) return true;
    // the decode-shaped kernel loads its row before it knows whether the record is dropped: fine for
    // one record, wasted reads for the dropped part of a batch under best effort (a replayable
    // step's policy is not known when it is captured)
    if (a.drop_newest || a.step) return false;
    return (uint64_t)nb * (a.listed_rows + 1u) <= 8192u;
}

// Element alignment of every source of a batch, and whether all of them allow 16-byte moves.
dmi_status_t check_batch_sources(uint32_t n, const void *const *data, uint32_t es, bool *all16)
{
    *all16 = true;
    for (uint32_t i = 0; i < n; i++) {
        if (!data[i]) return fail(DMI_ERR_INVALID_ARG, "data[%u] is NULL", i);
        if ((uintptr_t)data[i] % es) return fail(DMI_ERR_INVALID_ARG, "data[%u] is not element aligned", i);
        if ((uintptr_t)data[i] % 16u) *all16 = false;
    }
    return DMI_OK;
}

PlanEnv plan_env(const dmi_ring *r) { return PlanEnv{r->dev_ring, r->dev_cap, r->host_cap, r->dctrl, r->cfg.rank_tag, r}; }

dmi_status_t plan_capture(const PlanEnv &env, uint32_t point_id, const dmi_selection_t *sel, const dmi_transform_t *xf,
                          const Geometry &geo, CaptureArgs &a, Plan &pl, bool fixed_row_count_ok)
{
    const dmi_ring *r = env.masks;
    const uint32_t es_in = dtype_size(geo.src_dtype);
    uint64_t listed = 0;
    for (uint32_t i = 0; i < sel->n_reqs; i++) listed += sel->reqs[i].tok_count;
    const uint32_t unit_elems = geo.vec16 ? 16u / es_in : 1u;
    const uint64_t upr = geo.row_elems / unit_elems;
    if (listed > 0xFFFFFFFFull || listed * upr > 0xFFFFFFFFull)
        return fail(DMI_ERR_TOO_LARGE, "selection of %llu rows x %llu units exceeds one record",
                    (unsigned long long)listed, (unsigned long long)upr);
    const uint64_t ub = dmi_record_bytes(sel->n_reqs, listed, geo.row_elems, xf->out_dtype, xf->summary_mask);
    if (ub > env.cap)
        return fail(DMI_ERR_TOO_LARGE, "record of %llu bytes exceeds the device ring (%llu)",
                    (unsigned long long)ub, (unsigned long long)env.cap);
    if (env.host_cap && ub > env.host_cap)      // such a record could be drained but never polled whole
        return fail(DMI_ERR_TOO_LARGE, "record of %llu bytes exceeds the host ring (%llu)",
                    (unsigned long long)ub, (unsigned long long)env.host_cap);
    pl.listed = listed;
    pl.ub = ub;
    pl.rows_known = listed;
    pl.size_known = sel->keep_mask_dev == nullptr;
    if (fixed_row_count_ok && r &&  // (not for a replayable step: its keep vector changes between replays)
        sel->keep_mask_dev && sel->keep_mask_dev >= r->mask_buf && sel->keep_mask_dev < r->mask_buf + 4u * r->mask_stride &&
        (size_t)(sel->keep_mask_dev - r->mask_buf) % r->mask_stride == 0) {
        // a keep vector that came through dmi_set_keep_mask: the host knows what it holds, so
        // admission and accounting work with the record's real size instead of the bound
        const std::vector<uint8_t> &hm = r->mask_host[(size_t)(sel->keep_mask_dev - r->mask_buf) / r->mask_stride];
        if (hm.size() == sel->n_reqs) {
            uint64_t kept = 0;
            for (uint32_t i = 0; i < sel->n_reqs; i++) kept += hm[i] ? sel->reqs[i].tok_count : 0u;
            pl.ub = dmi_record_bytes(sel->n_reqs, kept, geo.row_elems, xf->out_dtype, xf->summary_mask);
            pl.rows_known = kept;
            pl.size_known = true;
        }
    }

    const bool index_mode = sel->row_index_dev != nullptr;
    bool one_row_each = true;
    for (uint32_t i = 0; one_row_each && i < sel->n_reqs; i++) one_row_each = sel->reqs[i].tok_count == 1u;
    const bool simple = one_row_each && sel->keep_mask_dev == nullptr;
    a.one_row_each = one_row_each ? 1u : 0u;
    a.listed_rows = (uint32_t)listed;
    const bool tab_lds = !simple && sel->n_reqs <= kLdsTableMax;
    a.n_seg = geo.n_seg;
    a.seg_units = geo.seg_elems / unit_elems;
    a.keep_mask = sel->keep_mask_dev;
    a.row_index = sel->row_index_dev;
    a.n_reqs = sel->n_reqs;
    a.src_dtype = geo.src_dtype;
    a.out_dtype = xf->out_dtype;
    a.summary_mask = xf->summary_mask;
    a.rec_flags = (a.paged ? DMI_REC_PAGED : 0u) | (sel->keep_mask_dev ? DMI_REC_MASKED : 0u) |
                  (index_mode ? DMI_REC_INDEXED : 0u);
    a.row_elems = geo.row_elems;
    a.units_per_row = (uint32_t)upr;
    // a wavefront per row when rows are short, or of moderate length and plentiful (no block-level
    // reduction, four rows in flight per workgroup); otherwise a workgroup per row
    a.rows_per_wg = (upr <= 128u || (upr <= 1024u && listed >= 2048u)) ? 4u : 1u;
    a.point_id = point_id;
    a.rank_tag = env.rank_tag;
    a.ring = env.ring;
    a.cap = env.cap;
    a.ctrl = env.ctrl;
    a.simple = simple ? 1u : 0u;
    auto shift_of = [](uint64_t v) { return v && (v & (v - 1u)) == 0 ? (uint32_t)__builtin_ctzll(v) : 32u; };
    a.upr_shift = shift_of(upr);
    a.bs_shift = shift_of(a.block_size);
    a.seg_shift = shift_of(a.seg_units);
    a.table_in_lds = tab_lds ? 1u : 0u;
    a.lds_bytes = capture_lds_bytes(simple ? 0u : sel->n_reqs, index_mode, tab_lds);

    pl.grid = plan_grid(a, 1u);

    // requests listing several rows take the decode-shaped kernel with one workgroup per listed
    // row: a launch whose row count must be able to change later (a replayable step) does not
    pl.decode = decode_kernel_applies(a, geo.vec16) && (one_row_each || fixed_row_count_ok);
    pl.row_map = pl.decode && !one_row_each && !index_mode;
    if (pl.decode) {
        // the host knows this record exactly: geometry and header travel as kernel arguments
        // (the kernel itself puts sequence number and step id into the header)
        const uint64_t table_bytes = pad64((uint64_t)sel->n_reqs * 16u);
        a.payload_bytes = listed * geo.row_elems * dtype_size(xf->out_dtype);
        a.off_payload = DMI_HEADER_BYTES + table_bytes;
        a.off_sum = a.off_payload + pad64(a.payload_bytes);
        a.sum_arr = pad64(listed * 4u);
        a.record_bytes = ub;
        a.rows_consecutive = sel->row_index_dev == nullptr && one_row_each;
        a.row_first = sel->reqs[0].row_base + sel->reqs[0].tok_start;
        for (uint32_t i = 1; a.rows_consecutive && i < sel->n_reqs; i++)
            a.rows_consecutive = sel->reqs[i].row_base + sel->reqs[i].tok_start == a.row_first + i;
        a.hdr[0] = DMI_MAGIC;
        a.hdr[1] = 1u | (DMI_HEADER_BYTES << 16);
        a.hdr[6] = point_id;
        a.hdr[7] = a.src_dtype | (a.out_dtype << 8) | (a.summary_mask << 16) | (a.rec_flags << 24);
        a.hdr[8] = sel->n_reqs;  a.hdr[9] = (uint32_t)listed;  a.hdr[10] = geo.row_elems;  a.hdr[11] = a.rank_tag;
        a.hdr[12] = (uint32_t)ub;               a.hdr[13] = (uint32_t)(ub >> 32);
        a.hdr[14] = (uint32_t)a.payload_bytes;  a.hdr[15] = (uint32_t)(a.payload_bytes >> 32);
    }
    return DMI_OK;
}

// Issue the captures of `n` tensors of one shape that share selection and transform (n = 1: an
// ordinary observe): as few launches as the ring and kMaxBatch allow, each of them producing
// the records, sequence numbers and counters that single launches in the same order would.
// points / srcs list the tensors that passed the gate; *n_launched counts how many of them
// have been issued when the call returns (all of them unless it fails).
dmi_status_t observe_common(dmi_ring *r, uint32_t n, const uint32_t *points, const uint8_t *const *srcs,
                            const dmi_selection_t *sel, const dmi_transform_t *xf, uint64_t step_id,
                            void *hip_stream, const Geometry &geo, CaptureArgs &a, uint32_t *n_launched)
{
    hipStream_t s = (hipStream_t)hip_stream;
    *n_launched = 0;
    if (r->step_open)
        return fail(DMI_ERR_INVALID_ARG, "a replayable step is between dmi_step_begin and dmi_step_end");
    Plan pl;
    dmi_status_t st = plan_capture(plan_env(r), points[0], sel, xf, geo, a, pl, true);
    if (st != DMI_OK) return st;
    const uint64_t ub = pl.ub;
    const uint32_t mode = r->mode.load(std::memory_order_relaxed);
    r->last_stream.store(hip_stream, std::memory_order_release);
    // a launch of several records lays them down one behind the other from one head: under the
    // completeness policy they must fit the ring together (the kernels rely on it), so a batch
    // that does not is issued in pieces, each waiting for its room as single observes would
    const uint64_t fit = r->dev_cap / ub < kMaxBatch ? r->dev_cap / ub : kMaxBatch;
    uint32_t slot = 0;
    bool staged = false, host_decides = false;
    BatchArgs b;
    memset(&b, 0, sizeof b);

    // one launch: records [first, first + cnt) of the caller's list; force_drop: they are records
    // the host already knows cannot fit, launched with one workgroup each only to be counted; tail:
    // as many records behind the cnt launched ones that the host knows cannot fit either, counted
    // by the same launch without any workgroup of their own
    auto issue = [&](uint32_t first, uint32_t cnt, uint64_t floor, bool force_drop, uint32_t tail) -> dmi_status_t {
        dmi_status_t rc;
        if ((rc = commit_slot_room(r, cnt + tail)) != DMI_OK) return rc;
        if (!staged) {
            if ((rc = stage_selection(r, sel, a.paged != 0, pl.row_map, s, &slot)) != DMI_OK) return rc;
            staged = true;
        }
        const uint64_t seq = r->next_seq.load(std::memory_order_relaxed);
        a.req_table = reinterpret_cast<const uint4 *>(r->slab + (size_t)slot * r->slab_slot_words);
        a.row0 = r->slab + (size_t)slot * r->slab_slot_words + 4u * (size_t)sel->n_reqs;
        a.row_map = pl.row_map ? a.row0 + sel->n_reqs : nullptr;
        a.seq = seq;
        a.n_batch = cnt;
        a.step_id = step_id;
        a.cslot = &r->dctrl->slots[(seq + cnt + tail - 1u) % kCommitSlots];
        a.tail_floor = floor;
        a.drop_newest = mode == DMI_POLICY_DROP_NEWEST ? 1u : 0u;
        a.force_drop = force_drop ? 1u : 0u;
        a.n_tail_drop = tail;
        // best effort: every fourth launch refreshes the drained-up-to mark from the host's word
        // (a read across the host link by one lane); in between, the launch-time floor stands
        a.tail_src = (a.drop_newest && (r->launches.load(std::memory_order_relaxed) & 3u) == 0) ? r->htail_dev : nullptr;
        a.par_in = r->chain_par;
        a.step = nullptr;
        a.node = 0;
        for (uint32_t i = 0; i < cnt; i++) b.src[i] = srcs[first + i];
        for (uint32_t i = 0; i < cnt + tail; i++) b.point[i] = points[first + i];

        // (only the general kernel counts a tail)
        const bool decode = !force_drop && !tail && pl.decode && batch_takes_decode_kernel(a, cnt);
        const uint32_t grid = force_drop ? 1u : cnt == 1u ? pl.grid : plan_grid(a, cnt);
        const hipError_t e = decode ? launch_capture_decode(a, b, s) : launch_capture(a, b, grid, geo.vec16, s);
        if (e != hipSuccess) return fail(DMI_ERR_HIP, "capture launch failed: %s", hipGetErrorString(e));
        const uint64_t bytes = force_drop ? 0u : ub * cnt;      // what the launch may add to the ring
        // can the host tell what this launch does?  Under the completeness policy nothing is dropped;
        // under best effort the caller of this function has decided (host_decides) which records fit
        const bool exact = pl.size_known && (mode == DMI_POLICY_BLOCK || host_decides);
        r->chain_par ^= 1u;
        r->last_launch_ns.store(now_ns(), std::memory_order_relaxed);
        {
            std::lock_guard<std::mutex> lk(r->pmu);
            r->launches.fetch_add(1, std::memory_order_relaxed);
            r->next_seq.store(seq + cnt + tail, std::memory_order_release);
            if (exact && !force_drop) {
                r->window.bytes += bytes; r->window.records += cnt; r->window.rows += pl.rows_known * cnt;
                r->window.drop_bytes += ub * tail; r->window.drop_records += tail;
                r->window.drop_rows += pl.rows_known * tail;
            } else if (exact) {
                r->window.drop_bytes += ub * (cnt + tail); r->window.drop_records += cnt + tail;
                r->window.drop_rows += pl.rows_known * (cnt + tail);
            } else {
                r->window_exact = false;
            }
        }
        if (exact && r->head_exact) r->exact_head += bytes;
        else r->head_exact = false;
        r->inflight.emplace_back(seq + cnt + tail - 1u, bytes);    // confirmed launch by launch: the last record stands for all
        r->inflight_sum += bytes;
        r->unprobed_launches += 1;
        r->unprobed_bytes += bytes;
        return DMI_OK;
    };

    for (uint32_t done = 0; done < n;) {
        uint32_t nb = n - done < kMaxBatch ? n - done : kMaxBatch;
        uint32_t n_keep = nb;
        if (mode == DMI_POLICY_BLOCK) {
            if (nb > fit) nb = (uint32_t)fit;
            n_keep = nb;
            if ((st = wait_for_room(r, ub * nb)) != DMI_OK) return st;
        } else {
            head_upper_bound(r);    // keeps the in-flight list short
        }
        const uint64_t floor = r->drain_done.load(std::memory_order_acquire);
        host_decides = false;
        if (mode == DMI_POLICY_DROP_NEWEST && pl.size_known) {
            // Best effort: while the host knows where the head will stand when this launch runs, it
            // knows which records fit, because the kernel decides on this very drained mark or a newer
            // one (a newer one only makes more room).  It then launches the records that fit as
            // usual and the ones that do not apart, with a single workgroup each, only to be counted:
            // under sustained overload those are a third or more of all records, and a full grid of
            // workgroups for each of them, all finding out that they have nothing to do, costs a
            // quarter of what copying the record would.  And since the outcome is known, the host
            // needs no commit slot fetched to follow the head (an event behind the launches will do).
            // Not while the host runs far ahead of the GPU, though: the drained mark it decides on is
            // the one of this moment, the kernel's is at most a launch or so older than its own start.
            if ((st = advance_commits(r, false)) != DMI_OK) return st;
            if (!r->head_exact &&
                r->confirmed.load(std::memory_order_acquire) == r->next_seq.load(std::memory_order_relaxed)) {
                r->head_exact = true;
                r->exact_head = r->committed.load(std::memory_order_acquire);
            }
            constexpr uint64_t kTightLaunches = 4;
            const bool tight = r->launches.load(std::memory_order_relaxed) -
                               r->confirmed_launches.load(std::memory_order_acquire) <= kTightLaunches;
            if (r->head_exact && tight) {
                host_decides = true;
                const uint64_t used = r->exact_head - floor;
                const uint64_t room = used < r->dev_cap ? (r->dev_cap - used) / ub : 0u;
                if (room < nb) n_keep = (uint32_t)room;
            }
        }
        // (a tail is only ever the host's own decision: sizes known, so the launch's outcome is exact)
        // (nothing fits: one workgroup counts them all)
        if (n_keep) st = issue(done, n_keep, floor, false, nb - n_keep);
        else st = issue(done, 1u, floor, true, nb - 1u);
        if (st != DMI_OK) return st;
        done += nb;
        *n_launched = done;
        if (r->unprobed_launches >= 16u || r->unprobed_bytes >= r->probe_bytes) {
            r->unprobed_launches = 0;
            r->unprobed_bytes = 0;
            if ((st = record_probe(r)) != DMI_OK) return st;
        }
    }
    return DMI_OK;
}

// Common front gate: argument checks shared by all observes.
dmi_status_t gate_args(dmi_ring *r, const dmi_selection_t *sel, const dmi_transform_t *xf, uint32_t src_dtype)
{
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    if (!sel || !xf) return fail(DMI_ERR_INVALID_ARG, "selection / transform is NULL");
    if (sel->n_reqs > r->max_reqs)
        return fail(DMI_ERR_INVALID_ARG, "n_reqs %u exceeds max_reqs_per_observe %u", sel->n_reqs, r->max_reqs);
    if (sel->n_reqs && !sel->reqs) return fail(DMI_ERR_INVALID_ARG, "reqs is NULL");
    if (!transform_ok(src_dtype, xf->out_dtype))
        return fail(DMI_ERR_INVALID_ARG, "unsupported dtype pair %u -> %u", src_dtype, xf->out_dtype);
    if (xf->summary_mask & ~7u) return fail(DMI_ERR_INVALID_ARG, "bad summary_mask %u", xf->summary_mask);
    return DMI_OK;
}

// Hook filtering and sampling for one observation (arguments already checked).
// Returns DMI_OK to proceed, a positive code to stop without error.
dmi_status_t gate_point(dmi_ring *r, uint32_t point_id, const dmi_selection_t *sel, uint64_t step_id)
{
    r->observed_calls++;
    if (r->point_off[point_id]) { r->disabled_calls++; return DMI_POINT_DISABLED; }
    const uint32_t k = r->sample_k.load(std::memory_order_relaxed);
    if (step_id % k != r->sample_phase.load(std::memory_order_relaxed)) {
        uint64_t listed = 0;
        for (uint32_t i = 0; i < sel->n_reqs; i++) listed += sel->reqs[i].tok_count;
        r->sampled_out_calls++;
        r->sampled_out_rows += listed;
        return DMI_SAMPLED_OUT;
    }
    return DMI_OK;
}

dmi_status_t gate(dmi_ring *r, uint32_t point_id, const dmi_selection_t *sel, const dmi_transform_t *xf,
                  uint64_t step_id, uint32_t src_dtype)
{
    dmi_status_t st = gate_args(r, sel, xf, src_dtype);
    if (st != DMI_OK) return st;
    if (point_id >= DMI_MAX_POINTS) return fail(DMI_ERR_INVALID_ARG, "point_id %u >= %u", point_id, DMI_MAX_POINTS);
    return gate_point(r, point_id, sel, step_id);
}

// The gate for a batch: every tensor passes it on its own, in order, exactly as if it had been
// observed alone.  live[] receives the positions that go on to be captured.
dmi_status_t gate_batch(dmi_ring *r, uint32_t n, const uint32_t *point_ids, const void *const *data,
                        const dmi_selection_t *sel, const dmi_transform_t *xf, uint64_t step_id, uint32_t src_dtype,
                        std::vector<uint32_t> &live, dmi_status_t *all_stopped)
{
    dmi_status_t st = gate_args(r, sel, xf, src_dtype);
    if (st != DMI_OK) return st;
    if (n && (!point_ids || !data)) return fail(DMI_ERR_INVALID_ARG, "point_ids / data is NULL");
    for (uint32_t i = 0; i < n; i++)
        if (point_ids[i] >= DMI_MAX_POINTS)
            return fail(DMI_ERR_INVALID_ARG, "point_ids[%u] = %u >= %u", i, point_ids[i], DMI_MAX_POINTS);
    live.clear();
    *all_stopped = DMI_POINT_DISABLED;
    for (uint32_t i = 0; i < n; i++) {
        const dmi_status_t g = gate_point(r, point_ids[i], sel, step_id);
        if (g == DMI_OK) live.push_back(i);
        else if (g == DMI_SAMPLED_OUT) *all_stopped = DMI_SAMPLED_OUT;
    }
    return DMI_OK;
}

// The library's drain thread (section 4.3): follows the commits and issues a batch of copies once
// enough has accumulated by any of four measures: committed bytes, committed records, how full the
// device ring is, how long the oldest waiting byte has waited.
void bg_loop(dmi_ring *r)
{
    (void)hipSetDevice(r->dev);
    const uint64_t min_bytes = r->cfg.bg_min_bytes ? r->cfg.bg_min_bytes : (1u << 20);
    const uint64_t min_records = r->cfg.bg_min_records ? r->cfg.bg_min_records : 64u;
    const uint64_t occupancy_pct = r->cfg.bg_occupancy_pct ? r->cfg.bg_occupancy_pct : 50u;
    const uint64_t timeout_ns = (uint64_t)(r->cfg.bg_timeout_us ? r->cfg.bg_timeout_us : 200u) * 1000ull;
    // how long the producer must have paused before this thread puts a probe of its own behind
    // its launches (while it keeps launching it probes by itself)
    const uint64_t quiet_ns = timeout_ns < 200000ull ? timeout_ns : 200000ull;
    uint64_t waiting_since = 0, last_probe = 0;
    while (!r->stop.load(std::memory_order_acquire)) {
        if (r->quiet.load(std::memory_order_acquire)) {
            // a stream capture is open on the producer's side: stay away from the HIP API
            r->bg_parked.store(true, std::memory_order_release);
            std::this_thread::sleep_for(std::chrono::microseconds(50));
            continue;
        }
        r->bg_parked.store(false, std::memory_order_release);
        bool idle_probes;
        {
            std::lock_guard<std::mutex> lk(r->pmu);
            idle_probes = r->probes.empty();
        }
        // every probe is a barrier, or a small launch, in the inference queue
        if (idle_probes && now_ns() - last_probe >= quiet_ns &&
            now_ns() - r->last_launch_ns.load(std::memory_order_relaxed) >= quiet_ns) {
            (void)record_probe(r);
            last_probe = now_ns();
        }
        (void)advance_commits(r, false);
        uint64_t pending_bytes, pending_records, undrained;
        {
            std::lock_guard<std::mutex> lk(r->mu);
            // copies issued by somebody's non-blocking dmi_drain are noted here as they finish: with
            // this thread running, nobody else looks at the drain stream
            (void)reap(r, false);
            uint64_t committed, committed_records;
            {
                std::lock_guard<std::mutex> pk(r->pmu);
                committed = read_committed(r);
                committed_records = r->snap[0];
            }
            pending_bytes = committed - r->drain_issued;
            pending_records = pending_bytes ? committed_records - r->drain_issued_records : 0u;
            undrained = committed - r->drain_done.load(std::memory_order_relaxed);
        }
        const uint64_t t = now_ns();
        if (pending_bytes == 0) waiting_since = 0;
        else if (!waiting_since) waiting_since = t;
        const bool by_bytes = pending_bytes >= min_bytes;
        const bool by_records = pending_records >= min_records;
        const bool by_occupancy = pending_bytes && undrained * 100u >= occupancy_pct * r->dev_cap;
        const bool by_timeout = pending_bytes && t - waiting_since >= timeout_ns;
        if (by_bytes || by_records || by_occupancy || by_timeout) {
            uint64_t moved = 0;
            (void)drain(r, true, &moved);
            waiting_since = 0;
            if (moved) continue;
        }
        std::this_thread::sleep_for(std::chrono::microseconds(20));
    }
}

void free_ring(dmi_ring *r)
{
    if (!r) return;
    if (r->drain_stream) { (void)hipStreamSynchronize(r->drain_stream); (void)hipStreamDestroy(r->drain_stream); }
    if (r->ctl_stream) { (void)hipStreamSynchronize(r->ctl_stream); (void)hipStreamDestroy(r->ctl_stream); }
    if (r->htail) (void)hipHostFree((void *)r->htail);
    for (auto &p : r->probes) (void)hipEventDestroy(p.ev);
    for (auto ev : r->probe_pool) (void)hipEventDestroy(ev);
    if (r->dev_ring) (void)hipFree(r->dev_ring);
    if (r->dctrl) (void)hipFree(r->dctrl);
    if (r->slab) (void)hipFree(r->slab);
    if (r->mask_buf) (void)hipFree(r->mask_buf);
    if (r->host_ring) (void)hipHostFree(r->host_ring);
    if (r->hslots) (void)hipHostFree((void *)r->hslots);
    delete r;
}


}  // namespace host
}  // namespace dmi

// =========================================================================== C ABI
extern "C" {

const char *dmi_last_error(void) { return last_error_cstr(); }
const char *dmi_version(void) { return "dmi-ring 0.1 (gfx950)"; }

uint64_t dmi_record_bytes(uint32_t n_reqs, uint64_t n_rows, uint32_t row_elems, uint32_t out_dtype,
                          uint32_t summary_mask)
{
    uint64_t b = DMI_HEADER_BYTES;
    b += pad64((uint64_t)n_reqs * 16u);
    b += pad64(n_rows * row_elems * dtype_size(out_dtype));
    b += (uint64_t)__builtin_popcount(summary_mask & 7u) * pad64(n_rows * 4u);
    return b;
}

dmi_status_t dmi_ring_create(const dmi_ring_config_t *cfg, dmi_ring_t **out)
{
    if (!cfg || !out) return fail(DMI_ERR_INVALID_ARG, "cfg / out is NULL");
    if (cfg->device_ring_bytes < 4096 || cfg->host_ring_bytes < 4096 || cfg->device_ring_bytes % 64 ||
        cfg->host_ring_bytes % 64)
        return fail(DMI_ERR_INVALID_ARG, "ring sizes must be multiples of 64 and at least 4096");
    if ((cfg->flags & DMI_DRAIN_COPY_ENGINE) && (cfg->flags & DMI_DRAIN_KERNEL))
        return fail(DMI_ERR_INVALID_ARG, "choose one drain mode");
    // DMI_DRAIN_MODE=kernel|copy in the environment overrides the drain engine (for comparisons
    // without touching the caller's code)
    uint32_t flags = cfg->flags;
    if (const char *m = getenv("DMI_DRAIN_MODE")) {
        if (!strcmp(m, "kernel")) flags = (flags & ~(uint32_t)DMI_DRAIN_COPY_ENGINE) | DMI_DRAIN_KERNEL;
        else if (!strcmp(m, "copy")) flags = (flags & ~(uint32_t)DMI_DRAIN_KERNEL) | DMI_DRAIN_COPY_ENGINE;
        else return fail(DMI_ERR_INVALID_ARG, "DMI_DRAIN_MODE must be 'kernel' or 'copy'");
    }
    const uint32_t max_reqs = cfg->max_reqs_per_observe ? cfg->max_reqs_per_observe : 1024u;
    if (max_reqs > 4096u) return fail(DMI_ERR_INVALID_ARG, "max_reqs_per_observe > 4096");
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess || n_dev <= 0)
        return fail(DMI_ERR_HIP, "no HIP device available (%s)", hipGetErrorString(e));
    if (cfg->device_id < 0 || cfg->device_id >= n_dev) return fail(DMI_ERR_INVALID_ARG, "bad device_id");
    HIP_TRY(hipSetDevice(cfg->device_id));

    dmi_ring *r = new (std::nothrow) dmi_ring;
    if (!r) return fail(DMI_ERR_NOMEM, "out of host memory");
    r->cfg = *cfg;
    r->cfg.flags = flags;
    r->dev = cfg->device_id;
    r->dev_cap = cfg->device_ring_bytes;
    r->host_cap = cfg->host_ring_bytes;
    r->max_reqs = max_reqs;
    r->block_timeout_ms = cfg->block_timeout_ms ? cfg->block_timeout_ms : 2000u;
    r->point_off.assign(DMI_MAX_POINTS, 0);
    r->slab_slot_words = (max_reqs * 5u + kDecodeMaxListed + 63u) & ~63u;
    // a probe at least every 16 launches, or every 1/32 of the ring (not under 8 MiB): often enough
    // for the drain to follow closely, rare enough that its cost in the producer's stream stays small
    r->probe_bytes = r->dev_cap / 32u > (8u << 20) ? r->dev_cap / 32u : (8u << 20);

    auto bail = [&](hipError_t err, const char *what) {
        fail(DMI_ERR_HIP, "%s failed: %s", what, hipGetErrorString(err));
        free_ring(r);
        return DMI_ERR_HIP;
    };
    if ((e = hipMalloc((void **)&r->dev_ring, r->dev_cap)) != hipSuccess) return bail(e, "hipMalloc(device ring)");
    if ((e = hipMalloc((void **)&r->dctrl, sizeof(DevCtrl))) != hipSuccess) return bail(e, "hipMalloc(ctrl)");
    if ((e = hipMalloc((void **)&r->slab, (size_t)kSlabSlots * r->slab_slot_words * 4u)) != hipSuccess)
        return bail(e, "hipMalloc(selection slab)");
    r->mask_stride = (max_reqs + 255u) & ~255u;
    if ((e = hipMalloc((void **)&r->mask_buf, (size_t)4u * r->mask_stride)) != hipSuccess)
        return bail(e, "hipMalloc(keep vectors)");
    if ((e = hipHostMalloc((void **)&r->host_ring, r->host_cap, hipHostMallocMapped)) != hipSuccess)
        return bail(e, "hipHostMalloc(host ring)");
    if ((e = hipHostGetDevicePointer((void **)&r->host_ring_dev, r->host_ring, 0)) != hipSuccess)
        return bail(e, "hipHostGetDevicePointer(host ring)");
    // touch every page now: the consumer's first read of a page should not pay for a fault
    memset(r->host_ring, 0, r->host_cap);
    if ((e = hipHostMalloc((void **)&r->hslots, sizeof(CommitSlot) * kCommitSlots,
                           hipHostMallocMapped | hipHostMallocCoherent)) != hipSuccess)
        return bail(e, "hipHostMalloc(commit slots)");
    if ((e = hipHostGetDevicePointer((void **)&r->hslots_dev, (void *)r->hslots, 0)) != hipSuccess)
        return bail(e, "hipHostGetDevicePointer(commit slots)");
    memset((void *)r->hslots, 0, sizeof(CommitSlot) * kCommitSlots);
    {
        DevCtrl *init = new (std::nothrow) DevCtrl;
        if (!init) { free_ring(r); return fail(DMI_ERR_NOMEM, "out of host memory"); }
        memset(init, 0, sizeof *init);
        e = hipMemcpy(r->dctrl, init, sizeof *init, hipMemcpyHostToDevice);
        delete init;
        if (e != hipSuccess) return bail(e, "hipMemcpy(ctrl)");
    }
    if ((e = hipHostMalloc((void **)&r->htail, 64, hipHostMallocMapped | hipHostMallocCoherent)) != hipSuccess)
        return bail(e, "hipHostMalloc(tail word)");
    if ((e = hipHostGetDevicePointer((void **)&r->htail_dev, (void *)r->htail, 0)) != hipSuccess)
        return bail(e, "hipHostGetDevicePointer(tail word)");
    *r->htail = 0;
    if ((e = hipStreamCreateWithFlags(&r->drain_stream, hipStreamNonBlocking)) != hipSuccess)
        return bail(e, "hipStreamCreate");
    if ((e = hipStreamCreateWithFlags(&r->ctl_stream, hipStreamNonBlocking)) != hipSuccess)
        return bail(e, "hipStreamCreate");
    if ((e = hipDeviceSynchronize()) != hipSuccess) return bail(e, "hipDeviceSynchronize");
    if (flags & DMI_BG_THREAD) r->bg = std::thread(bg_loop, r);
    *out = r;
    return DMI_OK;
}

dmi_status_t dmi_ring_destroy(dmi_ring_t *r)
{
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    (void)hipSetDevice(r->dev);
    (void)dmi_exporter_stop(r);
    r->stop.store(true, std::memory_order_release);
    if (r->bg.joinable()) r->bg.join();
    free_ring(r);
    return DMI_OK;
}

}  // extern "C"

namespace dmi {
namespace host {

// Checks of a selection against a dense source of T rows (not in index mode, where the
// kernel checks every index itself).
dmi_status_t check_dense_rows(const dmi_req_sel_t *reqs, uint32_t n, int64_t T)
{
    for (uint32_t i = 0; i < n; i++) {
        const dmi_req_sel_t &q = reqs[i];
        if (!q.tok_count) continue;
        const uint64_t last = (uint64_t)q.row_base + q.tok_start + (uint64_t)(q.tok_count - 1u) * q.tok_step;
        if (last >= (uint64_t)T)
            return fail(DMI_ERR_INVALID_ARG, "request %u selects row %llu of a %lld-row tensor", i,
                        (unsigned long long)last, (long long)T);
    }
    return DMI_OK;
}

// Same for a paged source: block-table row and token positions.
dmi_status_t check_paged_rows(const dmi_req_sel_t *reqs, uint32_t n, uint32_t n_seqs, uint32_t block_size,
                              int64_t bt_stride)
{
    for (uint32_t i = 0; i < n; i++) {
        const dmi_req_sel_t &q = reqs[i];
        if (q.row_base >= n_seqs) return fail(DMI_ERR_INVALID_ARG, "request %u: block-table row out of range", i);
        if (!q.tok_count) continue;
        const uint64_t last = (uint64_t)q.tok_start + (uint64_t)(q.tok_count - 1u) * q.tok_step;
        if (last > 0x7FFFFFFFull || last / block_size >= (uint64_t)bt_stride)
            return fail(DMI_ERR_INVALID_ARG, "request %u: token %llu is beyond the block table", i,
                        (unsigned long long)last);
    }
    return DMI_OK;
}

// Validate a dense tensor + selection and fill the source part of the kernel arguments.
dmi_status_t prep_dense(const dmi_tensor_t *t, const dmi_selection_t *sel, Geometry &geo, CaptureArgs &a)
{
    const uint32_t es = dtype_size(t->dtype);
    const int64_t T = t->shape[0], E = t->shape[1];
    if (T < 0 || T > 0xFFFFFFFFll || E < 1 || E > 0x7FFFFFFF) return fail(DMI_ERR_INVALID_ARG, "bad tensor shape");
    if ((E > 1 && t->stride[1] != 1) || t->stride[0] < 0) return fail(DMI_ERR_INVALID_ARG, "bad tensor stride");
    if (!t->data && T > 0) return fail(DMI_ERR_INVALID_ARG, "tensor data is NULL");
    if ((uintptr_t)t->data % es) return fail(DMI_ERR_INVALID_ARG, "tensor data is not element aligned");
    if (!sel->row_index_dev) {
        dmi_status_t st = check_dense_rows(sel->reqs, sel->n_reqs, T);
        if (st != DMI_OK) return st;
    }
    geo.src_dtype = t->dtype;
    geo.row_elems = (uint32_t)E;
    geo.n_seg = 1;
    geo.seg_elems = (uint32_t)E;
    geo.vec16 = (uintptr_t)t->data % 16 == 0 && ((uint64_t)t->stride[0] * es) % 16 == 0 && ((uint64_t)E * es) % 16 == 0;
    memset(&a, 0, sizeof a);
    a.src = (const uint8_t *)t->data;
    a.row_stride_b = t->stride[0] * (int64_t)es;
    a.n_src_rows = T;
    a.paged = 0;
    a.block_size = 1;
    return DMI_OK;
}

// Validate a paged KV description + selection and fill the source part of the kernel arguments.
dmi_status_t prep_paged(const dmi_paged_kv_t *kv, const dmi_selection_t *sel, Geometry &geo, CaptureArgs &a)
{
    const uint32_t es = dtype_size(kv->dtype);
    if (sel->row_index_dev) return fail(DMI_ERR_INVALID_ARG, "row_index_dev is not valid for paged captures");
    if (!kv->base || !kv->block_table_dev) return fail(DMI_ERR_INVALID_ARG, "kv base / block table is NULL");
    if (!kv->block_size || !kv->head_dim || !kv->n_heads || !kv->n_blocks || !kv->n_seqs)
        return fail(DMI_ERR_INVALID_ARG, "kv geometry has a zero field");
    if (kv->n_heads_sel < 1 || kv->n_heads_sel > DMI_MAX_HEADS_SEL)
        return fail(DMI_ERR_INVALID_ARG, "n_heads_sel must be 1..%u", DMI_MAX_HEADS_SEL);
    for (uint32_t i = 0; i < kv->n_heads_sel; i++)
        if (kv->heads_sel[i] >= kv->n_heads) return fail(DMI_ERR_INVALID_ARG, "selected head out of range");
    if (kv->block_stride < 0 || kv->slot_stride < 0 || kv->head_stride < 0 || kv->block_table_stride < 1)
        return fail(DMI_ERR_INVALID_ARG, "negative kv stride");
    if ((uintptr_t)kv->base % es) return fail(DMI_ERR_INVALID_ARG, "kv base is not element aligned");
    if ((uint64_t)kv->n_heads_sel * kv->head_dim > 0x7FFFFFFFull) return fail(DMI_ERR_INVALID_ARG, "row too long");
    {
        dmi_status_t st = check_paged_rows(sel->reqs, sel->n_reqs, kv->n_seqs, kv->block_size, kv->block_table_stride);
        if (st != DMI_OK) return st;
    }
    geo.src_dtype = kv->dtype;
    geo.n_seg = kv->n_heads_sel;
    geo.seg_elems = kv->head_dim;
    geo.row_elems = kv->n_heads_sel * kv->head_dim;
    geo.vec16 = (uintptr_t)kv->base % 16 == 0 && ((uint64_t)kv->block_stride * es) % 16 == 0 &&
                ((uint64_t)kv->slot_stride * es) % 16 == 0 && ((uint64_t)kv->head_stride * es) % 16 == 0 &&
                ((uint64_t)kv->head_dim * es) % 16 == 0;
    memset(&a, 0, sizeof a);
    a.src = (const uint8_t *)kv->base;
    a.n_src_rows = kv->n_blocks;
    a.block_stride_b = kv->block_stride * (int64_t)es;
    a.slot_stride_b = kv->slot_stride * (int64_t)es;
    a.head_stride_b = kv->head_stride * (int64_t)es;
    a.block_table = kv->block_table_dev;
    a.bt_stride = kv->block_table_stride;
    a.block_size = kv->block_size;
    for (uint32_t i = 0; i < kv->n_heads_sel; i++) a.heads_sel[i] = kv->heads_sel[i];
    a.paged = 1;
    return DMI_OK;
}

}  // namespace host
}  // namespace dmi

extern "C" {

dmi_status_t dmi_observe(dmi_ring_t *r, uint32_t point_id, const dmi_tensor_t *t, const dmi_selection_t *sel,
                         const dmi_transform_t *xf, uint64_t step_id, void *hip_stream)
{
    if (!t) return fail(DMI_ERR_INVALID_ARG, "tensor is NULL");
    dmi_status_t g = gate(r, point_id, sel, xf, step_id, t->dtype);
    if (g != DMI_OK) return g;
    Geometry geo;
    CaptureArgs a;
    if ((g = prep_dense(t, sel, geo, a)) != DMI_OK) return g;
    (void)hipSetDevice(r->dev);
    uint32_t launched = 0;
    return observe_common(r, 1u, &point_id, &a.src, sel, xf, step_id, hip_stream, geo, a, &launched);
}

dmi_status_t dmi_observe_paged(dmi_ring_t *r, uint32_t point_id, const dmi_paged_kv_t *kv,
                               const dmi_selection_t *sel, const dmi_transform_t *xf, uint64_t step_id,
                               void *hip_stream)
{
    if (!kv) return fail(DMI_ERR_INVALID_ARG, "kv is NULL");
    dmi_status_t g = gate(r, point_id, sel, xf, step_id, kv->dtype);
    if (g != DMI_OK) return g;
    Geometry geo;
    CaptureArgs a;
    if ((g = prep_paged(kv, sel, geo, a)) != DMI_OK) return g;
    (void)hipSetDevice(r->dev);
    uint32_t launched = 0;
    return observe_common(r, 1u, &point_id, &a.src, sel, xf, step_id, hip_stream, geo, a, &launched);
}

}  // extern "C"

namespace {

// The batch entry points behind their argument checks: gate every tensor, capture the ones
// that pass.  `first` is the source the geometry was prepared from (its alignment is checked
// with the others here).
dmi_status_t observe_batch(dmi_ring *r, uint32_t n, const uint32_t *point_ids, const void *const *data,
                           const dmi_selection_t *sel, const dmi_transform_t *xf, uint64_t step_id, void *hip_stream,
                           Geometry &geo, CaptureArgs &a, uint32_t *n_done)
{
    std::vector<uint32_t> live;
    dmi_status_t stopped = DMI_OK;
    dmi_status_t g = gate_batch(r, n, point_ids, data, sel, xf, step_id, geo.src_dtype, live, &stopped);
    if (g != DMI_OK) return g;
    if (live.empty()) {
        if (n_done) *n_done = n;
        return n ? stopped : DMI_OK;
    }
    std::vector<uint32_t> pts(live.size());
    std::vector<const uint8_t *> srcs(live.size());
    for (size_t k = 0; k < live.size(); k++) {
        pts[k] = point_ids[live[k]];
        srcs[k] = static_cast<const uint8_t *>(data[live[k]]);
    }
    (void)hipSetDevice(r->dev);
    uint32_t launched = 0;
    g = observe_common(r, (uint32_t)live.size(), pts.data(), srcs.data(), sel, xf, step_id, hip_stream, geo, a,
                       &launched);
    // positions of the caller's arrays dealt with: everything in front of the first tensor not yet issued
    if (n_done) *n_done = launched == live.size() ? n : live[launched];
    return g;
}

}  // namespace

extern "C" {

dmi_status_t dmi_observe_batch(dmi_ring_t *r, uint32_t n, const uint32_t *point_ids, const void *const *data,
                               const dmi_tensor_t *like, const dmi_selection_t *sel, const dmi_transform_t *xf,
                               uint64_t step_id, void *hip_stream, uint32_t *n_done)
{
    if (n_done) *n_done = 0;
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    if (!like) return fail(DMI_ERR_INVALID_ARG, "tensor description is NULL");
    if (!sel || !xf) return fail(DMI_ERR_INVALID_ARG, "selection / transform is NULL");
    if (n && (!point_ids || !data)) return fail(DMI_ERR_INVALID_ARG, "point_ids / data is NULL");
    if (!n) return DMI_OK;
    dmi_tensor_t t = *like;
    t.data = data[0];
    Geometry geo;
    CaptureArgs a;
    dmi_status_t g = prep_dense(&t, sel, geo, a);
    if (g != DMI_OK) return g;
    bool all16 = true;
    if ((g = check_batch_sources(n, data, dtype_size(t.dtype), &all16)) != DMI_OK) return g;
    geo.vec16 = geo.vec16 && all16;
    return observe_batch(r, n, point_ids, data, sel, xf, step_id, hip_stream, geo, a, n_done);
}

dmi_status_t dmi_observe_paged_batch(dmi_ring_t *r, uint32_t n, const uint32_t *point_ids, const void *const *bases,
                                     const dmi_paged_kv_t *like, const dmi_selection_t *sel,
                                     const dmi_transform_t *xf, uint64_t step_id, void *hip_stream, uint32_t *n_done)
{
    if (n_done) *n_done = 0;
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    if (!like) return fail(DMI_ERR_INVALID_ARG, "kv description is NULL");
    if (!sel || !xf) return fail(DMI_ERR_INVALID_ARG, "selection / transform is NULL");
    if (n && (!point_ids || !bases)) return fail(DMI_ERR_INVALID_ARG, "point_ids / bases is NULL");
    if (!n) return DMI_OK;
    dmi_paged_kv_t kv = *like;
    kv.base = bases[0];
    Geometry geo;
    CaptureArgs a;
    dmi_status_t g = prep_paged(&kv, sel, geo, a);
    if (g != DMI_OK) return g;
    bool all16 = true;
    if ((g = check_batch_sources(n, bases, dtype_size(kv.dtype), &all16)) != DMI_OK) return g;
    geo.vec16 = geo.vec16 && all16;
    return observe_batch(r, n, point_ids, bases, sel, xf, step_id, hip_stream, geo, a, n_done);
}

dmi_status_t dmi_drain(dmi_ring_t *r, uint32_t flags, uint64_t *bytes_moved)
{
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    (void)hipSetDevice(r->dev);
    if (bytes_moved) *bytes_moved = 0;
    const bool wait = !(flags & DMI_DRAIN_NONBLOCK);
    dmi_status_t st;
    if (!(flags & DMI_DRAIN_FLUSH)) {
        bool idle_probes;
        {
            std::lock_guard<std::mutex> lk(r->pmu);
            idle_probes = r->probes.empty();
        }
        if (idle_probes && (st = record_probe(r)) != DMI_OK) return st;
        if ((st = advance_commits(r, false)) != DMI_OK) return st;
        return drain(r, wait, bytes_moved);
    }
    // flush: everything issued so far must finish, then all of it is moved
    const uint64_t want_seq = r->next_seq.load(std::memory_order_acquire);
    if ((st = record_probe(r)) != DMI_OK) return st;
    const uint64_t t0 = now_ns();
    uint64_t total = 0, target = UINT64_MAX;
    for (;;) {
        if ((st = advance_commits(r, false)) != DMI_OK) return st;
        // once the launches issued before the call are known to have finished, their records lie
        // below the head committed at that moment: the call is done when the drain has passed it,
        // whatever a producer thread commits behind it in the meantime
        if (target == UINT64_MAX && r->confirmed.load(std::memory_order_acquire) >= want_seq)
            target = read_committed(r);
        uint64_t moved = 0;
        bool host_full = false;
        if ((st = drain(r, true, &moved, &host_full)) != DMI_OK) return st;
        total += moved;
        if (bytes_moved) *bytes_moved = total;
        if (target != UINT64_MAX && r->drain_done.load(std::memory_order_acquire) >= target) return DMI_OK;
        if (moved) continue;
        if (target != UINT64_MAX && host_full)
            return fail(DMI_ERR_AGAIN, "host ring is full: release records and drain again");
        if (now_ns() - t0 > (uint64_t)r->block_timeout_ms * 1000000ull)
            return fail(DMI_ERR_AGAIN, target == UINT64_MAX ? "observes did not finish within %u ms"
                                                            : "the drain did not finish within %u ms",
                        r->block_timeout_ms);
        std::this_thread::sleep_for(std::chrono::microseconds(10));
    }
}

dmi_status_t dmi_poll_host(dmi_ring_t *r, dmi_record_view_t *out, uint32_t max, uint32_t *n)
{
    if (!r || !n || (max && !out)) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    if (r->exp_running.load()) return fail(DMI_ERR_INVALID_ARG, "the exporter is this ring's consumer");
    return poll_host_impl(r, out, max, n);
}

}  // extern "C"

namespace dmi {
namespace host {
dmi_status_t poll_host_impl(dmi_ring *r, dmi_record_view_t *out, uint32_t max, uint32_t *n)
{
    *n = 0;
    std::lock_guard<std::mutex> lk(r->mu);
    // with the library's drain thread running, arrivals are noted by that thread; a HIP call
    // on the drain stream's events from here would queue up behind its blocking wait
    if (!(r->cfg.flags & DMI_BG_THREAD) && !r->quiet.load(std::memory_order_acquire)) {
        dmi_status_t st = reap(r, false);
        if (st != DMI_OK) return st;
    }
    const uint64_t done = r->drain_done.load(std::memory_order_acquire);
    while (*n < max && r->poll_cursor + DMI_HEADER_BYTES <= done) {
        const uint64_t off = r->poll_cursor % r->host_cap;
        const uint8_t *h = r->host_ring + off;      // capacities and records are multiples of 64
        uint32_t magic;
        uint64_t seq, rb;
        memcpy(&magic, h, 4);
        memcpy(&seq, h + 8, 8);
        memcpy(&rb, h + 48, 8);
        if (magic != DMI_MAGIC || rb < DMI_HEADER_BYTES || rb % 64 || rb > r->dev_cap)
            return fail(DMI_ERR_CLOSED, "corrupt record header at stream offset %llu",
                        (unsigned long long)r->poll_cursor);
        if (r->poll_cursor + rb > done) break;
        dmi_record_view_t &v = out[*n];
        v.p0 = h;
        v.n0 = rb < r->host_cap - off ? rb : r->host_cap - off;
        v.n1 = rb - v.n0;
        v.p1 = v.n1 ? r->host_ring : nullptr;
        v.seq = seq;
        r->polled.emplace_back(seq, r->poll_cursor + rb);
        r->poll_cursor += rb;
        ++*n;
    }
    return DMI_OK;
}

dmi_status_t release_host_impl(dmi_ring *r, uint64_t upto)
{
    std::lock_guard<std::mutex> lk(r->mu);
    while (!r->polled.empty() && r->polled.front().first <= upto) {
        r->released_bytes += r->polled.front().second - r->released;
        r->released = r->polled.front().second;
        r->polled.pop_front();
    }
    return DMI_OK;
}
}  // namespace host
}  // namespace dmi

extern "C" {

dmi_status_t dmi_release_host(dmi_ring_t *r, uint64_t upto)
{
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    if (r->exp_running.load()) return fail(DMI_ERR_INVALID_ARG, "the exporter is this ring's consumer");
    return release_host_impl(r, upto);
}

dmi_status_t dmi_set_policy(dmi_ring_t *r, const dmi_policy_t *p)
{
    if (!r || !p) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    if (p->mode > DMI_POLICY_DROP_NEWEST || p->sample_k < 1 || p->sample_phase >= p->sample_k)
        return fail(DMI_ERR_INVALID_ARG, "bad policy");
    r->mode.store(p->mode);
    r->sample_k.store(p->sample_k);
    r->sample_phase.store(p->sample_phase);
    return DMI_OK;
}

dmi_status_t dmi_policy_select(uint32_t strategy, const dmi_req_info_t *reqs, uint32_t n, uint64_t bytes_per_row,
                               uint64_t budget, uint8_t *keep, uint32_t *n_kept)
{
    if (strategy > DMI_SELECT_KEEP_BY_PATTERN) return fail(DMI_ERR_INVALID_ARG, "unknown selection strategy");
    if (n && (!reqs || !keep)) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    std::vector<uint32_t> order(n);
    for (uint32_t i = 0; i < n; i++) order[i] = i;
    const bool by_pattern = strategy == DMI_SELECT_KEEP_BY_PATTERN;
    std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
        if (by_pattern) {
            const bool mx = reqs[x].matches != 0, my = reqs[y].matches != 0;
            if (mx != my) return mx;
        }
        return reqs[x].admit_order < reqs[y].admit_order;
    });
    uint64_t used = 0;
    uint32_t kept = 0;
    bool open = true;       // a prefix: once a request does not fit, nothing after it is kept
    for (uint32_t k = 0; k < n; k++) {
        const uint32_t i = order[k];
        const unsigned __int128 cost = (unsigned __int128)reqs[i].rows * bytes_per_row;
        if (open && cost <= (unsigned __int128)(budget - used)) {
            used += (uint64_t)cost;
            keep[i] = 1;
            kept++;
        } else {
            open = false;
            keep[i] = 0;
        }
    }
    if (n_kept) *n_kept = kept;
    return DMI_OK;
}

dmi_status_t dmi_ring_free_bytes(dmi_ring_t *r, uint64_t *free_bytes)
{
    if (!r || !free_bytes) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    (void)hipSetDevice(r->dev);
    dmi_status_t st = advance_commits(r, false);
    if (st != DMI_OK) return st;
    const uint64_t used = head_upper_bound(r) - r->drain_done.load(std::memory_order_acquire);
    *free_bytes = used < r->dev_cap ? r->dev_cap - used : 0;
    return DMI_OK;
}

dmi_status_t dmi_set_keep_mask(dmi_ring_t *r, const uint8_t *keep, uint32_t n, void *hip_stream,
                               const uint8_t **keep_mask_dev)
{
    if (!r || !keep_mask_dev || (n && !keep)) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    if (n > r->max_reqs) return fail(DMI_ERR_INVALID_ARG, "n_reqs %u exceeds max_reqs_per_observe %u", n, r->max_reqs);
    (void)hipSetDevice(r->dev);
    const uint32_t which = r->mask_rr++ % 4u;
    uint8_t *dst = r->mask_buf + (size_t)which * r->mask_stride;
    r->mask_host[which].assign(keep, keep + n);
    std::vector<uint32_t> words((n + 3u) / 4u, 0u);
    if (n) memcpy(words.data(), keep, n);
    if (n) HIP_TRY(launch_upload(reinterpret_cast<uint32_t *>(dst), words.data(), (uint32_t)words.size(),
                                 (hipStream_t)hip_stream));
    *keep_mask_dev = dst;
    return DMI_OK;
}

dmi_status_t dmi_point_enable(dmi_ring_t *r, uint32_t point_id, int enabled)
{
    if (!r || point_id >= DMI_MAX_POINTS) return fail(DMI_ERR_INVALID_ARG, "bad ring / point_id");
    r->point_off[point_id] = enabled ? 0 : 1;
    return DMI_OK;
}

dmi_status_t dmi_get_stats(dmi_ring_t *r, dmi_stats_t *o)
{
    if (!r || !o) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    memset(o, 0, sizeof *o);
    o->observed_calls = r->observed_calls;
    o->launched_records = r->next_seq.load();
    (void)hipSetDevice(r->dev);
    (void)advance_commits(r, false);
    {
        std::lock_guard<std::mutex> lk(r->pmu);
        o->captured_records = r->snap[0];
        o->captured_rows = r->snap[1];
        o->captured_bytes = r->snap[2];
        o->dropped_records = r->snap[3];
        o->dropped_rows = r->snap[4];
        o->dropped_bytes = r->snap[5];
    }
    o->sampled_out_calls = r->sampled_out_calls;
    o->sampled_out_rows = r->sampled_out_rows;
    o->disabled_calls = r->disabled_calls;
    o->drained_bytes = r->drained_bytes;
    o->released_bytes = r->released_bytes;
    o->drain_batches = r->drain_batches;
    o->block_wait_ns = r->block_wait_ns;
    o->dev_ring_high_water = r->dev_high;
    o->host_ring_high_water = r->host_high;
    {
        std::lock_guard<std::mutex> lk(r->mu);
        uint64_t bad = 0;
        HIP_TRY(hipMemcpyAsync(&bad, &r->dctrl->bad_rows, 8, hipMemcpyDeviceToHost, r->ctl_stream));
        HIP_TRY(hipStreamSynchronize(r->ctl_stream));
        o->bad_rows = bad;
    }
    return DMI_OK;
}

dmi_status_t dmi_get_point_drops(dmi_ring_t *r, uint32_t point_id, uint64_t *n)
{
    if (!r || !n || point_id >= DMI_MAX_POINTS) return fail(DMI_ERR_INVALID_ARG, "bad argument");
    (void)hipSetDevice(r->dev);
    uint32_t v = 0;
    std::lock_guard<std::mutex> lk(r->mu);
    HIP_TRY(hipMemcpyAsync(&v, &r->dctrl->point_drops[point_id], 4, hipMemcpyDeviceToHost, r->ctl_stream));
    HIP_TRY(hipStreamSynchronize(r->ctl_stream));
    *n = v;
    return DMI_OK;
}

dmi_status_t dmi_debug_fill_rings(dmi_ring_t *r, uint8_t value)
{
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    (void)hipSetDevice(r->dev);
    std::lock_guard<std::mutex> lk(r->mu);
    HIP_TRY(hipMemsetAsync(r->dev_ring, value, r->dev_cap, r->drain_stream));
    HIP_TRY(hipStreamSynchronize(r->drain_stream));
    memset(r->host_ring, value, r->host_cap);
    return DMI_OK;
}

}  // extern "C"
