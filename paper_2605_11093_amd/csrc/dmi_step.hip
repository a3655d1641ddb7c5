// Replayable steps (paper section 4.4, policy manager; section 4.1 on graph compatibility):
// capture launches that read sequence base, step id, tail floor and policy from device
// memory, so that they can sit in the caller's hipGraph.
#include "dmi_ring.h"

using namespace dmi;
using namespace dmi::host;

extern "C" {

// ------------------------------------------------------------------ replayable steps
dmi_status_t dmi_step_create(dmi_ring_t *r, uint32_t max_observes, dmi_step_t **out)
{
    if (!r || !out) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    if (max_observes < 1u || max_observes > DMI_STEP_MAX_OBSERVES)
        return fail(DMI_ERR_INVALID_ARG, "max_observes must be 1..%u", DMI_STEP_MAX_OBSERVES);
    (void)hipSetDevice(r->dev);
    dmi_step *st = new (std::nothrow) dmi_step;
    if (!st) return fail(DMI_ERR_NOMEM, "out of host memory");
    st->r = r;
    st->max_nodes = max_observes;
    hipError_t e = hipMalloc((void **)&st->dparams, sizeof(StepParams));
    if (e == hipSuccess) e = hipMalloc((void **)&st->slab, (size_t)max_observes * r->slab_slot_words * 4u);
    // a first launch out of this library, so that none of its code is loaded under a capture
    StepParams zero;
    memset(&zero, 0, sizeof zero);
    if (e == hipSuccess) e = launch_step_begin(r->dctrl, st->dparams, zero, 0u, 0u, nullptr, r->ctl_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(r->ctl_stream);
    if (e != hipSuccess) {
        if (st->dparams) (void)hipFree(st->dparams);
        if (st->slab) (void)hipFree(st->slab);
        delete st;
        return fail(DMI_ERR_HIP, "step setup failed: %s", hipGetErrorString(e));
    }
    *out = st;
    return DMI_OK;
}

dmi_status_t dmi_step_destroy(dmi_step_t *st)
{
    if (!st) return fail(DMI_ERR_INVALID_ARG, "step is NULL");
    if (st->open) st->r->quiet.store(0, std::memory_order_release);
    if (st->begun) st->r->step_open = false;
    (void)hipSetDevice(st->r->dev);
    (void)hipFree(st->dparams);
    (void)hipFree(st->slab);
    delete st;
    return DMI_OK;
}

dmi_status_t dmi_step_capture_begin(dmi_step_t *st)
{
    if (!st) return fail(DMI_ERR_INVALID_ARG, "step is NULL");
    if (st->open || st->sealed) return fail(DMI_ERR_INVALID_ARG, "the step is already open or sealed");
    dmi_ring *r = st->r;
    // the caller is about to capture a stream: the library's own threads must keep away from
    // the HIP API until dmi_step_seal (some of their calls would invalidate the capture)
    r->quiet.store(1, std::memory_order_release);
    if (r->bg.joinable()) {
        const uint64_t t0 = now_ns();
        while (!r->bg_parked.load(std::memory_order_acquire)) {
            if (now_ns() - t0 > 2000000000ull) {
                r->quiet.store(0, std::memory_order_release);
                return fail(DMI_ERR_AGAIN, "the drain thread did not pause");
            }
            std::this_thread::sleep_for(std::chrono::microseconds(50));
        }
    }
    st->open = true;
    return DMI_OK;
}
}  // extern "C"

namespace {

// Add the captures of n tensors of one shape to an open step (n = 1: one observe) and issue
// their launches, as few as kMaxBatch allows, on the capturing stream.  The only HIP calls made
// here are the capture-status query and the kernel launches.
dmi_status_t step_add(dmi_step *st, uint32_t n, const uint32_t *points, const uint8_t *const *srcs,
                      const dmi_selection_t *sel, const dmi_transform_t *xf, const Geometry &geo, CaptureArgs &a,
                      uint32_t n_seqs, void *hip_stream, uint32_t *node_out)
{
    dmi_ring *r = st->r;
    if (st->rec_launch.size() + n > st->max_nodes)
        return fail(DMI_ERR_INVALID_ARG, "the step would hold more than max_observes (%u) records", st->max_nodes);
    // outside a capture the launch would run at once, with whatever the parameter block holds
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)hip_stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusActive)
        return fail(DMI_ERR_INVALID_ARG, "hip_stream is not capturing");
    StepNode nd;
    dmi_status_t rc = plan_capture(plan_env(r), points[0], sel, xf, geo, a, nd.pl, false);
    if (rc != DMI_OK) return rc;

    // nodes captured with the same selection share one table (and are updated together)
    std::vector<uint32_t> words;
    selection_words(sel->reqs, sel->n_reqs, a.paged != 0, nd.pl.row_map, words);
    uint32_t ti = 0;
    for (; ti < st->tables.size(); ti++)
        if (st->tables[ti].paged == (a.paged != 0) && st->tables[ti].row_map == nd.pl.row_map &&
            st->tables[ti].words == words) break;
    if (ti == st->tables.size()) {
        StepTable t;
        t.words.swap(words);
        t.reqs.assign(sel->reqs, sel->reqs + sel->n_reqs);
        t.paged = a.paged != 0;
        t.row_map = nd.pl.row_map;
        t.slot = ti;                // at most one table per node, so slots suffice
        st->tables.push_back(std::move(t));
    }
    if (node_out) *node_out = (uint32_t)st->rec_launch.size();
    uint32_t *slot = st->slab + (size_t)st->tables[ti].slot * r->slab_slot_words;
    BatchArgs b;
    memset(&b, 0, sizeof b);
    for (uint32_t done = 0; done < n;) {
        const uint32_t nb = n - done < kMaxBatch ? n - done : kMaxBatch;
        const uint32_t launch = (uint32_t)st->nodes.size(), first_rec = (uint32_t)st->rec_launch.size();
        a.req_table = reinterpret_cast<const uint4 *>(slot);
        a.row0 = slot + 4u * (size_t)sel->n_reqs;
        a.row_map = nd.pl.row_map ? a.row0 + sel->n_reqs : nullptr;
        a.seq = 0;
        a.n_batch = nb;
        a.step_id = 0;
        a.cslot = nullptr;
        a.tail_floor = 0;
        a.drop_newest = 0;
        a.tail_src = nullptr;           // the device copy that the step's begin launch refreshes
        a.par_in = launch & 1u;         // dmi_step_begin leaves head and tail in copy 0
        a.step = st->dparams;
        a.node = first_rec;             // sequence number of the launch's first record, relative to the step's
        for (uint32_t i = 0; i < nb; i++) { b.src[i] = srcs[done + i]; b.point[i] = points[done + i]; }
        const bool decode = nd.pl.decode && batch_takes_decode_kernel(a, nb);
        const hipError_t e = decode ? launch_capture_decode(a, b, (hipStream_t)hip_stream)
                                    : launch_capture(a, b, plan_grid(a, nb), geo.vec16, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail(DMI_ERR_HIP, "capture launch failed: %s", hipGetErrorString(e));
        nd.a = a;
        nd.first_rec = first_rec;
        nd.n_batch = nb;
        nd.geo = geo;
        nd.xf = *xf;
        nd.point_id = points[done];
        nd.table = ti;
        nd.index_mode = sel->row_index_dev != nullptr;
        nd.masked = sel->keep_mask_dev != nullptr;
        nd.n_seqs = n_seqs;
        st->nodes.push_back(nd);
        st->rec_launch.insert(st->rec_launch.end(), nb, launch);
        done += nb;
    }
    return DMI_OK;
}

// Front checks of dmi_step_observe*: state, arguments, hook filtering (a disabled point
// adds no launch to the step: it is not in the graph at all).
dmi_status_t step_gate(dmi_step *st, uint32_t n, const uint32_t *point_ids, const dmi_selection_t *sel,
                       const dmi_transform_t *xf, uint32_t src_dtype, std::vector<uint32_t> &live)
{
    if (!st) return fail(DMI_ERR_INVALID_ARG, "step is NULL");
    if (!st->open) return fail(DMI_ERR_INVALID_ARG, "call dmi_step_capture_begin first");
    dmi_ring *r = st->r;
    if (!sel || !xf) return fail(DMI_ERR_INVALID_ARG, "selection / transform is NULL");
    if (n && !point_ids) return fail(DMI_ERR_INVALID_ARG, "point_ids is NULL");
    for (uint32_t i = 0; i < n; i++)
        if (point_ids[i] >= DMI_MAX_POINTS)
            return fail(DMI_ERR_INVALID_ARG, "point_id %u >= %u", point_ids[i], DMI_MAX_POINTS);
    if (sel->n_reqs > r->max_reqs)
        return fail(DMI_ERR_INVALID_ARG, "n_reqs %u exceeds max_reqs_per_observe %u", sel->n_reqs, r->max_reqs);
    if (sel->n_reqs && !sel->reqs) return fail(DMI_ERR_INVALID_ARG, "reqs is NULL");
    if (!transform_ok(src_dtype, xf->out_dtype))
        return fail(DMI_ERR_INVALID_ARG, "unsupported dtype pair %u -> %u", src_dtype, xf->out_dtype);
    if (xf->summary_mask & ~7u) return fail(DMI_ERR_INVALID_ARG, "bad summary_mask %u", xf->summary_mask);
    live.clear();
    for (uint32_t i = 0; i < n; i++)
        if (!r->point_off[point_ids[i]]) live.push_back(i);
    return live.empty() ? DMI_POINT_DISABLED : DMI_OK;
}

// The tensors of a batch whose points are enabled, and their captures added to the step.
dmi_status_t step_add_live(dmi_step *st, const std::vector<uint32_t> &live, const uint32_t *point_ids,
                           const void *const *data, const dmi_selection_t *sel, const dmi_transform_t *xf,
                           const Geometry &geo, CaptureArgs &a, uint32_t n_seqs, void *hip_stream, uint32_t *node)
{
    std::vector<uint32_t> pts(live.size());
    std::vector<const uint8_t *> srcs(live.size());
    for (size_t k = 0; k < live.size(); k++) {
        pts[k] = point_ids[live[k]];
        srcs[k] = static_cast<const uint8_t *>(data[live[k]]);
    }
    return step_add(st, (uint32_t)live.size(), pts.data(), srcs.data(), sel, xf, geo, a, n_seqs, hip_stream, node);
}

}  // namespace

extern "C" {

dmi_status_t dmi_step_observe(dmi_step_t *st, uint32_t point_id, const dmi_tensor_t *t, const dmi_selection_t *sel,
                              const dmi_transform_t *xf, void *hip_stream, uint32_t *node)
{
    if (!t) return fail(DMI_ERR_INVALID_ARG, "tensor is NULL");
    std::vector<uint32_t> live;
    dmi_status_t g = step_gate(st, 1u, &point_id, sel, xf, t->dtype, live);
    if (g != DMI_OK) return g;
    Geometry geo;
    CaptureArgs a;
    if ((g = prep_dense(t, sel, geo, a)) != DMI_OK) return g;
    return step_add(st, 1u, &point_id, &a.src, sel, xf, geo, a, 0u, hip_stream, node);
}

dmi_status_t dmi_step_observe_batch(dmi_step_t *st, uint32_t n, const uint32_t *point_ids, const void *const *data,
                                    const dmi_tensor_t *like, const dmi_selection_t *sel, const dmi_transform_t *xf,
                                    void *hip_stream, uint32_t *node)
{
    if (!like) return fail(DMI_ERR_INVALID_ARG, "tensor description is NULL");
    if (!n || !data) return fail(DMI_ERR_INVALID_ARG, "empty batch / data is NULL");
    std::vector<uint32_t> live;
    dmi_status_t g = step_gate(st, n, point_ids, sel, xf, like->dtype, live);
    if (g != DMI_OK) return g;
    dmi_tensor_t t = *like;
    t.data = data[0];
    Geometry geo;
    CaptureArgs a;
    if ((g = prep_dense(&t, sel, geo, a)) != DMI_OK) return g;
    bool all16 = true;
    if ((g = check_batch_sources(n, data, dtype_size(t.dtype), &all16)) != DMI_OK) return g;
    geo.vec16 = geo.vec16 && all16;
    return step_add_live(st, live, point_ids, data, sel, xf, geo, a, 0u, hip_stream, node);
}

dmi_status_t dmi_step_observe_paged(dmi_step_t *st, uint32_t point_id, const dmi_paged_kv_t *kv,
                                    const dmi_selection_t *sel, const dmi_transform_t *xf, void *hip_stream,
                                    uint32_t *node)
{
    if (!kv) return fail(DMI_ERR_INVALID_ARG, "kv is NULL");
    std::vector<uint32_t> live;
    dmi_status_t g = step_gate(st, 1u, &point_id, sel, xf, kv->dtype, live);
    if (g != DMI_OK) return g;
    Geometry geo;
    CaptureArgs a;
    if ((g = prep_paged(kv, sel, geo, a)) != DMI_OK) return g;
    return step_add(st, 1u, &point_id, &a.src, sel, xf, geo, a, kv->n_seqs, hip_stream, node);
}

dmi_status_t dmi_step_observe_paged_batch(dmi_step_t *st, uint32_t n, const uint32_t *point_ids,
                                          const void *const *bases, const dmi_paged_kv_t *like,
                                          const dmi_selection_t *sel, const dmi_transform_t *xf, void *hip_stream,
                                          uint32_t *node)
{
    if (!like) return fail(DMI_ERR_INVALID_ARG, "kv description is NULL");
    if (!n || !bases) return fail(DMI_ERR_INVALID_ARG, "empty batch / bases is NULL");
    std::vector<uint32_t> live;
    dmi_status_t g = step_gate(st, n, point_ids, sel, xf, like->dtype, live);
    if (g != DMI_OK) return g;
    dmi_paged_kv_t kv = *like;
    kv.base = bases[0];
    Geometry geo;
    CaptureArgs a;
    if ((g = prep_paged(&kv, sel, geo, a)) != DMI_OK) return g;
    bool all16 = true;
    if ((g = check_batch_sources(n, bases, dtype_size(kv.dtype), &all16)) != DMI_OK) return g;
    geo.vec16 = geo.vec16 && all16;
    return step_add_live(st, live, point_ids, bases, sel, xf, geo, a, kv.n_seqs, hip_stream, node);
}

dmi_status_t dmi_step_seal(dmi_step_t *st)
{
    if (!st) return fail(DMI_ERR_INVALID_ARG, "step is NULL");
    if (!st->open) return fail(DMI_ERR_INVALID_ARG, "the step is not open");
    st->open = false;
    st->sealed = true;
    st->sum_ub = st->sum_listed = 0;
    for (auto &nd : st->nodes) { st->sum_ub += nd.pl.ub * nd.n_batch; st->sum_listed += nd.pl.listed * nd.n_batch; }
    st->r->quiet.store(0, std::memory_order_release);
    return DMI_OK;
}

dmi_status_t dmi_step_update(dmi_step_t *st, uint32_t node, const dmi_req_sel_t *reqs, uint32_t n_reqs)
{
    if (!st || !reqs) return fail(DMI_ERR_INVALID_ARG, "NULL argument");
    if (!st->sealed) return fail(DMI_ERR_INVALID_ARG, "the step is not sealed");
    if (st->begun) return fail(DMI_ERR_INVALID_ARG, "between dmi_step_begin and dmi_step_end");
    if (node >= st->rec_launch.size()) return fail(DMI_ERR_INVALID_ARG, "no node %u", node);
    dmi_ring *r = st->r;
    const uint32_t ti = st->nodes[st->rec_launch[node]].table;
    StepTable &tab = st->tables[ti];
    if (n_reqs != tab.reqs.size())
        return fail(DMI_ERR_INVALID_ARG, "the node was captured with %zu requests, not %u", tab.reqs.size(), n_reqs);
    uint64_t listed = 0;
    bool all_one = true;
    for (uint32_t i = 0; i < n_reqs; i++) { listed += reqs[i].tok_count; all_one = all_one && reqs[i].tok_count == 1u; }
    // every launch that reads this table must still be the launch that was captured
    std::vector<uint64_t> ubs;
    for (auto &nd : st->nodes) {
        if (nd.table != ti) continue;
        const CaptureArgs &a = nd.a;
        dmi_status_t rc = DMI_OK;
        if (a.paged) rc = check_paged_rows(reqs, n_reqs, nd.n_seqs, a.block_size, a.bt_stride);
        else if (!nd.index_mode) rc = check_dense_rows(reqs, n_reqs, a.n_src_rows);
        if (rc != DMI_OK) return rc;
        if ((a.simple || nd.pl.decode) && !all_one)
            return fail(DMI_ERR_INVALID_ARG, "captured with one row per request: capture the step again to change that");
        if (nd.pl.decode && a.rows_consecutive)
            for (uint32_t i = 0; i < n_reqs; i++)
                if (reqs[i].row_base + reqs[i].tok_start != a.row_first + i)
                    return fail(DMI_ERR_INVALID_ARG, "captured with request i in row %u + i: capture the step again "
                                                     "to change that", a.row_first);
        if (listed > 0xFFFFFFFFull || listed * a.units_per_row > 0xFFFFFFFFull)
            return fail(DMI_ERR_TOO_LARGE, "selection of %llu rows exceeds one record", (unsigned long long)listed);
        const uint64_t ub = dmi_record_bytes(n_reqs, listed, nd.geo.row_elems, nd.xf.out_dtype, nd.xf.summary_mask);
        if (ub > r->dev_cap)
            return fail(DMI_ERR_TOO_LARGE, "record of %llu bytes exceeds the device ring (%llu)",
                        (unsigned long long)ub, (unsigned long long)r->dev_cap);
        ubs.push_back(ub);
    }
    size_t k = 0;
    for (auto &nd : st->nodes) {
        if (nd.table != ti) continue;
        st->sum_ub += (ubs[k] - nd.pl.ub) * nd.n_batch;
        st->sum_listed += (listed - nd.pl.listed) * nd.n_batch;
        nd.pl.ub = ubs[k++];
        nd.pl.listed = listed;
    }
    tab.reqs.assign(reqs, reqs + n_reqs);
    selection_words(reqs, n_reqs, tab.paged, tab.row_map, tab.words);
    tab.dirty = true;
    return DMI_OK;
}

dmi_status_t dmi_step_begin(dmi_step_t *st, uint64_t step_id, void *hip_stream)
{
    if (!st) return fail(DMI_ERR_INVALID_ARG, "step is NULL");
    if (!st->sealed) return fail(DMI_ERR_INVALID_ARG, "the step is not sealed");
    dmi_ring *r = st->r;
    if (st->begun || r->step_open) return fail(DMI_ERR_INVALID_ARG, "a step is already between begin and end");
    (void)hipSetDevice(r->dev);
    hipStream_t s = (hipStream_t)hip_stream;
    const uint32_t n = (uint32_t)st->rec_launch.size();
    const uint32_t mode = r->mode.load(std::memory_order_relaxed);
    const uint32_t k = r->sample_k.load(std::memory_order_relaxed);
    const bool skip = step_id % k != r->sample_phase.load(std::memory_order_relaxed);
    dmi_status_t rc;
    r->last_stream.store(hip_stream, std::memory_order_release);
    if (!skip && n) {
        if (mode == DMI_POLICY_BLOCK) {
            // the flush before the forward step: the whole step must be sure to fit
            if (st->sum_ub > r->dev_cap)
                return fail(DMI_ERR_TOO_LARGE, "the step's records (%llu bytes) exceed the device ring (%llu): "
                            "launches inside a graph cannot wait for the drain",
                            (unsigned long long)st->sum_ub, (unsigned long long)r->dev_cap);
            if ((rc = wait_for_room(r, st->sum_ub)) != DMI_OK) return rc;
        } else {
            head_upper_bound(r);
        }
        if ((rc = commit_slot_room(r, n)) != DMI_OK) return rc;
    }
    for (auto &t : st->tables) {
        if (!t.dirty) continue;
        if (!t.words.empty())
            HIP_TRY(launch_upload(st->slab + (size_t)t.slot * r->slab_slot_words, t.words.data(),
                                  (uint32_t)t.words.size(), s));
        t.dirty = false;
    }
    StepParams v;
    v.seq_base = r->next_seq.load(std::memory_order_relaxed);
    v.step_id = step_id;
    v.tail_floor = r->drain_done.load(std::memory_order_acquire);
    v.flags = (mode == DMI_POLICY_DROP_NEWEST ? kStepDropNewest : 0u) | (skip ? kStepSkip : 0u);
    v.pad = 0;
    HIP_TRY(launch_step_begin(r->dctrl, st->dparams, v, r->chain_par, 0u,
                              mode == DMI_POLICY_DROP_NEWEST ? r->htail_dev : nullptr, s));
    r->chain_par = 0;
    st->seq_base = v.seq_base;
    st->skipped = skip;
    st->drop_newest = mode == DMI_POLICY_DROP_NEWEST;
    st->begun = true;
    r->step_open = true;
    r->observed_calls += n;
    if (skip) {
        r->sampled_out_calls += n;
        r->sampled_out_rows += st->sum_listed;
        return DMI_SAMPLED_OUT;
    }
    return DMI_OK;
}

dmi_status_t dmi_step_end(dmi_step_t *st, void *hip_stream)
{
    if (!st) return fail(DMI_ERR_INVALID_ARG, "step is NULL");
    if (!st->begun) return fail(DMI_ERR_INVALID_ARG, "dmi_step_begin has not been called");
    dmi_ring *r = st->r;
    (void)hipSetDevice(r->dev);
    const uint32_t n = (uint32_t)st->rec_launch.size();
    st->begun = false;
    r->step_open = false;
    r->chain_par = (uint32_t)st->nodes.size() & 1u;
    r->last_launch_ns.store(now_ns(), std::memory_order_relaxed);
    r->last_stream.store(hip_stream, std::memory_order_release);
    if (st->skipped || !n) return DMI_OK;
    for (auto &nd : st->nodes) {
        r->inflight.emplace_back(st->seq_base + nd.first_rec + nd.n_batch - 1u, nd.pl.ub * nd.n_batch);
        r->inflight_sum += nd.pl.ub * nd.n_batch;
    }
    // the step's launches decide drops and read keep vectors on the device
    bool host_knows = !st->drop_newest;
    for (auto &nd : st->nodes) host_knows = host_knows && !nd.masked;
    if (host_knows && r->head_exact) r->exact_head += st->sum_ub;
    else r->head_exact = false;
    {
        std::lock_guard<std::mutex> lk(r->pmu);
        r->launches.fetch_add(st->nodes.size(), std::memory_order_relaxed);
        r->next_seq.store(st->seq_base + n, std::memory_order_release);
        for (auto &nd : st->nodes) {
            if (st->drop_newest || nd.masked) { r->window_exact = false; break; }
            r->window.bytes += nd.pl.ub * nd.n_batch; r->window.records += nd.n_batch;
            r->window.rows += nd.pl.listed * nd.n_batch;
        }
    }
    r->unprobed_launches = 0;
    r->unprobed_bytes = 0;
    return record_probe(r);
}
}  // extern "C"
