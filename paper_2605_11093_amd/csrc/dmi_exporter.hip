// Exporter stages 2-3 (paper section 4.3): whole records out of the pinned ring into
// pageable memory (worker threads, committed in ring order), sliced per request.
#include "dmi_ring.h"

using namespace dmi;
using namespace dmi::host;

namespace {

// Wait for `pred` under `lk` for at most timeout_ms.  Against the system clock on purpose: that wait
// is pthread_cond_timedwait, which ThreadSanitizer follows; this libstdc++'s steady-clock wait is
// pthread_cond_clockwait, which it does not (it then believes the mutex held throughout the wait).
template <typename Pred>
bool wait_ms(std::condition_variable &cv, std::unique_lock<std::mutex> &lk, uint32_t timeout_ms, Pred pred)
{
    return cv.wait_until(lk, std::chrono::system_clock::now() + std::chrono::milliseconds(timeout_ms), pred);
}

// Pageable buffers are reused instead of allocated per record (section 4.3: the copy stage must keep
// up with the drain; a workload has few distinct record sizes, so nearly every record finds a buffer).
// A buffer serves a record of size s if s <= cap <= s + s/8.  Idle buffers count against the budget:
// in use + idle <= max_pageable_bytes (+ the 1/8 slack), the oldest idle ones are freed first.
// The pool has a lock of its own (pool_mu), taken last: the copy workers get their buffers without
// touching the lock that the consumer's queue is under.  The *_locked functions need pool_mu held.
uint8_t *pool_take_locked(dmi_ring *r, uint64_t size, uint64_t *cap)
{
    for (size_t i = r->exp_pool.size(); i-- > 0;) {         // newest first: most likely still in cache
        const PoolBuf b = r->exp_pool[i];
        if (b.cap >= size && b.cap <= size + size / 8) {
            r->exp_pool.erase(r->exp_pool.begin() + (ptrdiff_t)i);
            r->exp_pool_bytes -= b.cap;
            *cap = b.cap;
            return b.p;
        }
    }
    return nullptr;
}

void pool_trim_locked(dmi_ring *r, uint64_t keep_bytes)
{
    while (!r->exp_pool.empty() && r->exp_pool_bytes > keep_bytes) {
        r->exp_pool_bytes -= r->exp_pool.front().cap;
        free(r->exp_pool.front().p);
        r->exp_pool.erase(r->exp_pool.begin());
    }
}

// A record copy is done with: its budget share is free again, its buffer goes to the pool (emu held).
void retire_locked(dmi_ring *r, RecordCopy *rc)
{
    r->exp_bytes -= rc->size;
    std::lock_guard<std::mutex> pk(r->pool_mu);
    r->exp_pool.push_back(PoolBuf{rc->bytes, rc->cap});
    r->exp_pool_bytes += rc->cap;
    // a stopped exporter keeps nothing: slices given back after dmi_exporter_stop free their memory
    const bool keep = !r->exp_stop.load() && r->exp_max_bytes > r->exp_bytes;
    pool_trim_locked(r, keep ? r->exp_max_bytes - r->exp_bytes : 0);
    delete rc;
}

// A buffer for a record of `size` bytes: from the pool, else from the allocator.  If memory is short the
// idle buffers go first; after that the budget is the caller's promise that the record fits, so wait for
// the consumer to give copies back.
uint8_t *buffer_for(dmi_ring *r, uint64_t size, uint64_t *cap)
{
    for (;;) {
        {
            std::lock_guard<std::mutex> pk(r->pool_mu);
            if (uint8_t *p = pool_take_locked(r, size, cap)) { r->exp_reuses++; return p; }
        }
        if (uint8_t *p = static_cast<uint8_t *>(malloc(size))) { r->exp_mallocs++; *cap = size; return p; }
        {
            std::lock_guard<std::mutex> pk(r->pool_mu);
            if (!r->exp_pool.empty()) { pool_trim_locked(r, 0); continue; }
        }
        std::unique_lock<std::mutex> lk(r->emu);
        wait_ms(r->ecv_space, lk, 1, [] { return false; });
    }
}

// Exporter stage 3 for one record copy: shape / dtype from the header, one slice per request with rows.
void slice_record(RecordCopy *rc, std::vector<dmi_slice_t> &made)
{
    const uint8_t *b = rc->bytes;
    uint32_t n_reqs, n_rows, row_elems, point_id, rank_tag;
    uint64_t seq, step_id, payload_bytes;
    memcpy(&seq, b + 8, 8);
    memcpy(&step_id, b + 16, 8);
    memcpy(&point_id, b + 24, 4);
    memcpy(&n_reqs, b + 32, 4);
    memcpy(&n_rows, b + 36, 4);
    memcpy(&row_elems, b + 40, 4);
    memcpy(&rank_tag, b + 44, 4);
    memcpy(&payload_bytes, b + 56, 8);
    const uint32_t src_dtype = b[28], out_dtype = b[29], smask = b[30], flags = b[31];
    const uint64_t es = dtype_size(out_dtype);
    const uint8_t *table = b + DMI_HEADER_BYTES;
    const uint8_t *payload = table + pad64((uint64_t)n_reqs * 16u);
    const uint8_t *sums = payload + pad64(payload_bytes);
    const uint64_t sum_arr = pad64((uint64_t)n_rows * 4u);
    const float *arr[3] = {nullptr, nullptr, nullptr};
    {
        const uint8_t *p = sums;
        for (int bit = 0; bit < 3; bit++)
            if (smask & (1u << bit)) { arr[bit] = reinterpret_cast<const float *>(p); p += sum_arr; }
    }
    uint64_t row0 = 0;
    for (uint32_t q = 0; q < n_reqs; q++) {
        uint32_t e[4];
        memcpy(e, table + 16ull * q, 16);
        if (e[3] == 0) continue;
        dmi_slice_t sl;
        memset(&sl, 0, sizeof sl);
        sl.seq = seq; sl.step_id = step_id; sl.point_id = point_id; sl.rank_tag = rank_tag;
        sl.req_index = q; sl.req_id = e[0]; sl.tok_start = e[1]; sl.tok_step = e[2]; sl.n_rows = e[3];
        sl.row_elems = row_elems; sl.src_dtype = src_dtype; sl.out_dtype = out_dtype;
        sl.summary_mask = smask; sl.flags = flags;
        sl.rows = es ? payload + row0 * row_elems * es : nullptr;
        sl.l2 = arr[0] ? arr[0] + row0 : nullptr;
        sl.mean = arr[1] ? arr[1] + row0 : nullptr;
        sl.absmax = arr[2] ? arr[2] + row0 : nullptr;
        sl.owner = rc;
        made.push_back(sl);
        row0 += e[3];
    }
}

// Exporter copy worker: takes records (with a ticket in ring order) from the dispatcher,
// copies each into pageable memory, slices it, and commits the results in ticket order
// (the pinned space is given back in that order too).
void exporter_worker(dmi_ring *r)
{
    for (;;) {
        ExportJob job;
        {
            std::unique_lock<std::mutex> lk(r->jmu);
            r->jcv.wait(lk, [&] { return r->exp_stop.load() || !r->jobs.empty(); });
            if (r->jobs.empty()) return;        // stopping
            job = r->jobs.front();
            r->jobs.pop_front();
        }
        RecordCopy *rc = new RecordCopy;
        rc->size = job.view.n0 + job.view.n1;
        rc->bytes = buffer_for(r, rc->size, &rc->cap);
        memcpy(rc->bytes, job.view.p0, job.view.n0);
        if (job.view.n1) memcpy(rc->bytes + job.view.n0, job.view.p1, job.view.n1);
        std::vector<dmi_slice_t> made;
        slice_record(rc, made);
        rc->refs.store((uint32_t)made.size());
        r->exp_records++;
        r->exp_copied_bytes += rc->size;

        std::lock_guard<std::mutex> lk(r->emu);
        r->done_jobs.emplace(job.ticket, ExportDone{job.view.seq, rc, std::move(made)});
        bool any = false;
        while (!r->done_jobs.empty() && r->done_jobs.begin()->first == r->next_emit) {
            ExportDone &d = r->done_jobs.begin()->second;
            (void)release_host_impl(r, d.seq);      // pinned space is free again, in ring order
            if (d.slices.empty()) {                 // nothing to hand out: the copy goes at once
                retire_locked(r, d.rc);
                r->ecv_space.notify_all();
            } else {
                for (auto &sl : d.slices) r->slices.push_back(sl);
                any = true;
            }
            r->done_jobs.erase(r->done_jobs.begin());
            r->next_emit++;
        }
        if (any) r->ecv_data.notify_all();
    }
}

// Exporter dispatcher: polls whole records out of the pinned ring and hands them to the
// copy workers, bounded by the pageable budget (this is where back-pressure starts).
void exporter_loop(dmi_ring *r)
{
    (void)hipSetDevice(r->dev);
    dmi_record_view_t views[64];
    uint64_t ticket = 0;
    while (!r->exp_stop.load(std::memory_order_acquire)) {
        uint32_t n = 0;
        if (poll_host_impl(r, views, 64, &n) != DMI_OK || n == 0) {
            std::this_thread::sleep_for(std::chrono::microseconds(50));
            continue;
        }
        for (uint32_t i = 0; i < n; i++) {
            const uint64_t size = views[i].n0 + views[i].n1;
            {
                std::unique_lock<std::mutex> lk(r->emu);
                r->ecv_space.wait(lk, [&] {
                    return r->exp_stop.load() || r->exp_bytes == 0 || r->exp_bytes + size <= r->exp_max_bytes;
                });
                if (r->exp_stop.load()) return;
                r->exp_bytes += size;
            }
            {
                std::lock_guard<std::mutex> lk(r->jmu);
                r->jobs.push_back(ExportJob{views[i], ticket++});
            }
            r->jcv.notify_one();
        }
    }
}

}  // namespace

extern "C" {

dmi_status_t dmi_exporter_start(dmi_ring_t *r, uint64_t max_pageable_bytes, uint32_t n_copy_threads)
{
    if (!r || !max_pageable_bytes || n_copy_threads > 16u) return fail(DMI_ERR_INVALID_ARG, "bad argument");
    if (r->exp_running.exchange(true)) return fail(DMI_ERR_INVALID_ARG, "exporter already running");
    r->exp_stop.store(false);
    r->exp_max_bytes = max_pageable_bytes;
    r->next_emit = 0;
    const uint32_t n = n_copy_threads ? n_copy_threads : 3u;
    for (uint32_t i = 0; i < n; i++) r->exp_workers.emplace_back(exporter_worker, r);
    r->exporter = std::thread(exporter_loop, r);
    return DMI_OK;
}

dmi_status_t dmi_exporter_next(dmi_ring_t *r, dmi_slice_t *out, uint32_t timeout_ms)
{
    if (!r || !out) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    std::unique_lock<std::mutex> lk(r->emu);
    if (!wait_ms(r->ecv_data, lk, timeout_ms, [&] { return !r->slices.empty(); }))
        return fail(DMI_ERR_AGAIN, "no slice within %u ms", timeout_ms);
    *out = r->slices.front();
    r->slices.pop_front();
    return DMI_OK;
}

dmi_status_t dmi_exporter_next_many(dmi_ring_t *r, dmi_slice_t *out, uint32_t max, uint32_t *n, uint32_t timeout_ms)
{
    if (!r || !n || (max && !out)) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    *n = 0;
    std::unique_lock<std::mutex> lk(r->emu);
    if (!wait_ms(r->ecv_data, lk, timeout_ms, [&] { return !r->slices.empty(); }))
        return fail(DMI_ERR_AGAIN, "no slice within %u ms", timeout_ms);
    while (*n < max && !r->slices.empty()) {
        out[(*n)++] = r->slices.front();
        r->slices.pop_front();
    }
    return DMI_OK;
}

dmi_status_t dmi_exporter_release_many(dmi_ring_t *r, const dmi_slice_t *sl, uint32_t n)
{
    if (!r || (n && !sl)) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    for (uint32_t i = 0; i < n; i++) {
        dmi_status_t st = dmi_exporter_release(r, &sl[i]);
        if (st != DMI_OK) return st;
    }
    return DMI_OK;
}

dmi_status_t dmi_exporter_release(dmi_ring_t *r, const dmi_slice_t *sl)
{
    if (!r || !sl || !sl->owner) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    RecordCopy *rc = static_cast<RecordCopy *>(sl->owner);
    if (rc->refs.fetch_sub(1) == 1) {
        {
            std::lock_guard<std::mutex> lk(r->emu);
            retire_locked(r, rc);
        }
        r->ecv_space.notify_all();
    }
    return DMI_OK;
}

dmi_status_t dmi_debug_exporter_allocs(dmi_ring_t *r, uint64_t *allocated, uint64_t *reused)
{
    if (!r || !allocated || !reused) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    *allocated = r->exp_mallocs.load();
    *reused = r->exp_reuses.load();
    return DMI_OK;
}

dmi_status_t dmi_exporter_stop(dmi_ring_t *r)
{
    if (!r) return fail(DMI_ERR_INVALID_ARG, "ring is NULL");
    if (!r->exp_running.load()) return DMI_OK;
    {   // set under the lock the dispatcher evaluates its wait condition under
        std::lock_guard<std::mutex> lk(r->emu);
        r->exp_stop.store(true);
    }
    r->ecv_space.notify_all();
    if (r->exporter.joinable()) r->exporter.join();
    uint64_t dropped = 0;       // pageable budget booked for records no worker will copy
    {
        std::lock_guard<std::mutex> lk(r->jmu);
        for (auto &j : r->jobs) dropped += j.view.n0 + j.view.n1;
        r->jobs.clear();
    }
    r->jcv.notify_all();
    for (auto &w : r->exp_workers) if (w.joinable()) w.join();
    r->exp_workers.clear();
    {   // discard what was not handed out
        std::lock_guard<std::mutex> lk(r->emu);
        r->exp_bytes -= dropped;
        for (auto &kv : r->done_jobs) {
            if (kv.second.slices.empty()) {
                retire_locked(r, kv.second.rc);
            } else {
                for (auto &sl : kv.second.slices) r->slices.push_back(sl);
            }
        }
        r->done_jobs.clear();
        for (auto &sl : r->slices) {
            RecordCopy *rc = static_cast<RecordCopy *>(sl.owner);
            if (rc->refs.fetch_sub(1) == 1) retire_locked(r, rc);
        }
        r->slices.clear();
        std::lock_guard<std::mutex> pk(r->pool_mu);
        pool_trim_locked(r, 0);
    }
    r->exp_running.store(false);
    return DMI_OK;
}
}  // extern "C"
