// Multi-threaded exercise of the library's host runtime on the CPU stand-in runtime -- TEST
// INFRASTRUCTURE ONLY.  Built with -fsanitize=thread or -fsanitize=address by
// tests/test_host_runtime_sanitizers.py; exits 0 if every scenario's invariants hold (the
// sanitizers turn their own findings into a non-zero exit).
//
// Threads of a scenario, as include/dmi.h allows them: one producer (dmi_observe,
// dmi_observe_batch, replayable steps), the library's drain thread, one consumer
// (dmi_poll_host / dmi_release_host, or the exporter's queue), one thread reading dmi_get_stats,
// one thread issuing non-blocking and flushing drains.
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "dmi.h"
#include "dmi_debug.h"

#define CHECK(cond)                                                                          \
    do {                                                                                     \
        if (!(cond)) {                                                                       \
            fprintf(stderr, "%s:%d: CHECK failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, \
                    dmi_last_error());                                                       \
            exit(3);                                                                         \
        }                                                                                    \
    } while (0)

namespace {

struct Totals {
    std::atomic<uint64_t> records{0}, bytes{0}, slices{0};
    std::atomic<bool> producer_done{false};
};

uint64_t header_u64(const dmi_record_view_t &v, size_t off)
{
    uint64_t x;
    memcpy(&x, static_cast<const uint8_t *>(v.p0) + off, 8);
    return x;
}

// poll + release until the producer has finished and the ring is empty
void consumer_loop(dmi_ring_t *ring, Totals *t)
{
    uint64_t last_seq = UINT64_MAX;
    std::vector<dmi_record_view_t> views(64);
    int idle_after_done = 0;
    while (idle_after_done < 200) {
        uint32_t n = 0;
        CHECK(dmi_poll_host(ring, views.data(), (uint32_t)views.size(), &n) == DMI_OK);
        for (uint32_t i = 0; i < n; i++) {
            const dmi_record_view_t &v = views[i];
            CHECK(header_u64(v, 8) == v.seq);
            CHECK(header_u64(v, 48) == v.n0 + v.n1);
            CHECK(last_seq == UINT64_MAX || v.seq > last_seq);
            // the executor fills a record's payload with a byte derived from its sequence number
            const uint8_t want = (uint8_t)(0x40u + (v.seq & 0x3Fu));
            const uint8_t *tail = v.n1 ? static_cast<const uint8_t *>(v.p1) + v.n1 - 1
                                       : static_cast<const uint8_t *>(v.p0) + v.n0 - 1;
            CHECK(v.n0 + v.n1 <= 192 || *tail == want || *tail == 0);
            last_seq = v.seq;
            t->records++;
            t->bytes += v.n0 + v.n1;
        }
        if (n) CHECK(dmi_release_host(ring, views[n - 1].seq) == DMI_OK);
        else {
            if (t->producer_done.load()) idle_after_done++;
            std::this_thread::sleep_for(std::chrono::microseconds(50));
        }
    }
}

void exporter_consumer_loop(dmi_ring_t *ring, Totals *t)
{
    std::vector<dmi_slice_t> sl(256);
    uint64_t last_seq = 0;
    int idle_after_done = 0;
    while (idle_after_done < 100) {
        uint32_t n = 0;
        const dmi_status_t rc = dmi_exporter_next_many(ring, sl.data(), (uint32_t)sl.size(), &n, 2);
        CHECK(rc == DMI_OK || rc == DMI_ERR_AGAIN);
        for (uint32_t i = 0; i < n; i++) {
            CHECK(sl[i].seq >= last_seq);
            last_seq = sl[i].seq;
            if (sl[i].req_index == 0) t->records++;
            t->slices++;
        }
        if (n) CHECK(dmi_exporter_release_many(ring, sl.data(), n) == DMI_OK);
        else if (t->producer_done.load()) idle_after_done++;
    }
}

void stats_loop(dmi_ring_t *ring, Totals *t)
{
    dmi_stats_t prev;
    memset(&prev, 0, sizeof prev);
    while (!t->producer_done.load()) {
        dmi_stats_t s;
        CHECK(dmi_get_stats(ring, &s) == DMI_OK);
        CHECK(s.captured_records >= prev.captured_records && s.drained_bytes >= prev.drained_bytes);
        CHECK(s.released_bytes >= prev.released_bytes && s.released_bytes <= s.drained_bytes);
        CHECK(s.captured_records + s.dropped_records <= s.launched_records);
        prev = s;
        std::this_thread::sleep_for(std::chrono::microseconds(200));
    }
}

void drainer_loop(dmi_ring_t *ring, Totals *t)
{
    unsigned k = 0;
    while (!t->producer_done.load()) {
        uint64_t moved = 0;
        const dmi_status_t rc = dmi_drain(ring, (++k % 8 == 0) ? DMI_DRAIN_FLUSH : DMI_DRAIN_NONBLOCK, &moved);
        CHECK(rc == DMI_OK || rc == DMI_ERR_AGAIN);
        std::this_thread::sleep_for(std::chrono::microseconds(300));
    }
}

struct Source {
    std::vector<uint16_t> data;
    dmi_tensor_t t;
    Source(int64_t rows, int64_t cols) : data((size_t)(rows * cols), 0x3F80)
    {
        t.data = data.data(); t.dtype = DMI_DTYPE_BF16;
        t.shape[0] = rows; t.shape[1] = cols; t.stride[0] = cols; t.stride[1] = 1;
    }
};

void flush_all(dmi_ring_t *ring)
{
    for (int i = 0; i < 100000; i++) {
        const dmi_status_t rc = dmi_drain(ring, DMI_DRAIN_FLUSH, nullptr);
        if (rc == DMI_OK) return;
        CHECK(rc == DMI_ERR_AGAIN);
        std::this_thread::sleep_for(std::chrono::microseconds(100));
    }
    CHECK(!"the ring did not flush");
}

// one scenario: producer on this thread, the others beside it
void scenario(const char *name, uint32_t policy, bool use_exporter, bool with_steps, int n_iter)
{
    fprintf(stderr, "scenario %s\n", name);
    dmi_ring_config_t cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.device_ring_bytes = 1u << 20;
    cfg.host_ring_bytes = 2u << 20;
    cfg.flags = DMI_BG_THREAD;
    cfg.max_reqs_per_observe = 64;
    cfg.bg_min_bytes = 64u << 10;
    cfg.bg_timeout_us = 100;
    cfg.block_timeout_ms = 5;
    dmi_ring_t *ring = nullptr;
    CHECK(dmi_ring_create(&cfg, &ring) == DMI_OK);
    dmi_policy_t pol = {policy, 1, 0};
    CHECK(dmi_set_policy(ring, &pol) == DMI_OK);

    hipStream_t stream;
    CHECK(hipStreamCreate(&stream) == hipSuccess);
    Source a(64, 512), b(64, 512), c(64, 512);
    std::vector<dmi_req_sel_t> decode(16), ragged(3);
    for (uint32_t i = 0; i < 16; i++) decode[i] = {100 + i, i, 0, 1, 1};
    ragged[0] = {7, 0, 2, 5, 2}; ragged[1] = {8, 20, 0, 9, 1}; ragged[2] = {9, 63, 0, 1, 1};
    std::vector<uint8_t> keep = {1, 0, 1};
    const uint8_t *keep_dev = nullptr;
    const dmi_selection_t sel_decode = {16, decode.data(), nullptr, nullptr};
    const dmi_transform_t raw = {DMI_DTYPE_BF16, 0}, fp8_sum = {DMI_DTYPE_FP8_E4M3FN, DMI_SUM_L2 | DMI_SUM_ABSMAX};
    const uint32_t points[3] = {1, 2, 3};
    const void *datas[3] = {a.data.data(), b.data.data(), c.data.data()};

    // a replayable step of 3 launches (one of them a batch of 3), "captured" by the stand-in runtime
    dmi_step_t *step = nullptr;
    std::vector<FakeTask> graph;
    if (with_steps) {
        CHECK(dmi_step_create(ring, 8, &step) == DMI_OK);
        CHECK(dmi_step_capture_begin(step) == DMI_OK);
        fake_begin_capture(stream);
        uint32_t node = 99;
        CHECK(dmi_step_observe(step, 10, &a.t, &sel_decode, &raw, stream, &node) == DMI_OK && node == 0);
        CHECK(dmi_step_observe_batch(step, 3, points, datas, &a.t, &sel_decode, &fp8_sum, stream, &node) == DMI_OK);
        CHECK(node == 1);
        const dmi_selection_t sel_r = {3, ragged.data(), nullptr, nullptr};
        CHECK(dmi_step_observe(step, 11, &b.t, &sel_r, &raw, stream, &node) == DMI_OK && node == 4);
        graph = fake_end_capture(stream);
        CHECK(graph.size() == 3);
        CHECK(dmi_step_seal(step) == DMI_OK);
    }

    Totals tot;
    if (use_exporter) CHECK(dmi_exporter_start(ring, 8u << 20, 2) == DMI_OK);
    std::thread consumer(use_exporter ? exporter_consumer_loop : consumer_loop, ring, &tot);
    std::thread stats(stats_loop, ring, &tot);
    std::thread drainer(drainer_loop, ring, &tot);

    auto retry = [&](auto &&call) {
        for (int tries = 0; tries < 2000000; tries++) {
            const dmi_status_t rc = call();
            if (rc != DMI_ERR_AGAIN) return rc;
            std::this_thread::sleep_for(std::chrono::microseconds(20));     // the consumer is another thread
        }
        return (dmi_status_t)DMI_ERR_AGAIN;
    };
    for (int it = 0; it < n_iter; it++) {
        const uint64_t step_id = (uint64_t)it;
        if (it % 100 == 0) {            // the policy manager's knobs move while everything runs
            dmi_policy_t p2 = {policy, (it / 100) % 3 == 2 ? 2u : 1u, 0};
            CHECK(dmi_set_policy(ring, &p2) == DMI_OK);
            CHECK(dmi_point_enable(ring, 2, (it / 100) % 2 == 0) == DMI_OK);
        }
        CHECK(retry([&] { return dmi_observe(ring, 0, &a.t, &sel_decode, &raw, step_id, stream); }) >= 0);
        uint32_t done = 0, from = 0;
        CHECK(retry([&] {
                  const dmi_status_t rc = dmi_observe_batch(ring, 3 - from, points + from, datas + from, &a.t,
                                                            &sel_decode, &fp8_sum, step_id, stream, &done);
                  from += done;
                  return rc;
              }) >= 0);
        if (it % 3 == 0) {
            CHECK(dmi_set_keep_mask(ring, keep.data(), 3, stream, &keep_dev) == DMI_OK);
            const dmi_selection_t sel_k = {3, ragged.data(), keep_dev, nullptr};
            CHECK(retry([&] { return dmi_observe(ring, 4, &c.t, &sel_k, &raw, step_id, stream); }) >= 0);
        }
        if (with_steps && it % 2 == 1) {
            const dmi_status_t rc = retry([&] { return dmi_step_begin(step, step_id, stream); });
            CHECK(rc >= 0);
            fake_graph_launch(graph, stream);
            CHECK(dmi_step_end(step, stream) == DMI_OK);
        }
        if (it % 64 == 63) {
            uint64_t room = 0;
            CHECK(dmi_ring_free_bytes(ring, &room) == DMI_OK && room <= cfg.device_ring_bytes);
        }
    }
    CHECK(hipStreamSynchronize(stream) == hipSuccess);
    tot.producer_done.store(true);
    drainer.join();
    stats.join();
    if (!use_exporter) flush_all(ring);
    consumer.join();
    if (use_exporter) {
        // the exporter is the consumer: wait until it has taken everything that was captured
        for (int i = 0; i < 20000; i++) {
            dmi_stats_t s;
            CHECK(dmi_get_stats(ring, &s) == DMI_OK);
            if (s.captured_records + s.dropped_records == s.launched_records && s.released_bytes == s.captured_bytes) break;
            std::this_thread::sleep_for(std::chrono::microseconds(200));
            (void)dmi_drain(ring, DMI_DRAIN_NONBLOCK, nullptr);
        }
        CHECK(dmi_exporter_stop(ring) == DMI_OK);
        // the copy stage reuses its pageable buffers: far fewer allocations than records
        uint64_t allocated = 0, reused = 0;
        CHECK(dmi_debug_exporter_allocs(ring, &allocated, &reused) == DMI_OK);
        dmi_stats_t e;
        CHECK(dmi_get_stats(ring, &e) == DMI_OK);
        fprintf(stderr, "  exporter buffers: %llu allocated, %llu reused\n", (unsigned long long)allocated,
                (unsigned long long)reused);
        CHECK(allocated + reused == e.captured_records);
        if (e.captured_records > 64) CHECK(allocated * 4 < e.captured_records);
    }
    dmi_stats_t s;
    CHECK(dmi_get_stats(ring, &s) == DMI_OK);
    fprintf(stderr, "  launched %llu captured %llu dropped %llu drained %llu released %llu consumer saw %llu records\n",
            (unsigned long long)s.launched_records, (unsigned long long)s.captured_records,
            (unsigned long long)s.dropped_records, (unsigned long long)s.drained_bytes,
            (unsigned long long)s.released_bytes, (unsigned long long)tot.records.load());
    CHECK(s.captured_records + s.dropped_records == s.launched_records);
    CHECK(s.drained_bytes == s.captured_bytes && s.released_bytes == s.captured_bytes);
    if (policy == DMI_POLICY_BLOCK) CHECK(s.dropped_records == 0);
    if (!use_exporter) CHECK(tot.records.load() == s.captured_records && tot.bytes.load() == s.captured_bytes);
    uint64_t drops = 0, d = 0;
    for (uint32_t p : {0u, 1u, 2u, 3u, 4u, 10u, 11u}) { CHECK(dmi_get_point_drops(ring, p, &d) == DMI_OK); drops += d; }
    CHECK(drops == s.dropped_records);
    if (step) CHECK(dmi_step_destroy(step) == DMI_OK);
    CHECK(dmi_ring_destroy(ring) == DMI_OK);
    CHECK(hipStreamDestroy(stream) == hipSuccess);
}

// Best effort with the host knowing exactly where the head stands (everything flushed, nothing in
// flight): of a batch of six records into a ring that holds two and a half, the host launches the two
// that fit and has that launch count the four behind them; with the ring still full, the next batch
// is counted by a launch of one workgroup.  Single-threaded: what is checked is the bookkeeping.
void scenario_host_decided_drops()
{
    fprintf(stderr, "scenario drop-newest, the host decides\n");
    Source src(64, 512);
    std::vector<dmi_req_sel_t> decode(16);
    for (uint32_t i = 0; i < 16; i++) decode[i] = {100 + i, i, 0, 1, 1};
    const dmi_selection_t sel = {16, decode.data(), nullptr, nullptr};
    const dmi_transform_t raw = {DMI_DTYPE_BF16, 0};
    const uint64_t rb = dmi_record_bytes(16, 16, 512, DMI_DTYPE_BF16, 0);
    dmi_ring_config_t cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.device_ring_bytes = (2 * rb + rb / 2) / 64 * 64;
    cfg.host_ring_bytes = 1u << 20;
    cfg.max_reqs_per_observe = 64;
    dmi_ring_t *ring = nullptr;
    CHECK(dmi_ring_create(&cfg, &ring) == DMI_OK);
    dmi_policy_t pol = {DMI_POLICY_DROP_NEWEST, 1, 0};
    CHECK(dmi_set_policy(ring, &pol) == DMI_OK);
    hipStream_t stream;
    CHECK(hipStreamCreate(&stream) == hipSuccess);
    const uint32_t points[6] = {1, 2, 3, 4, 3, 2};
    const void *datas[6] = {src.data.data(), src.data.data(), src.data.data(), src.data.data(), src.data.data(), src.data.data()};
    uint32_t done = 0;
    CHECK(dmi_observe_batch(ring, 6, points, datas, &src.t, &sel, &raw, 0, stream, &done) == DMI_OK && done == 6);
    CHECK(dmi_observe_batch(ring, 6, points, datas, &src.t, &sel, &raw, 1, stream, &done) == DMI_OK && done == 6);
    CHECK(hipStreamSynchronize(stream) == hipSuccess);
    flush_all(ring);
    dmi_stats_t s;
    CHECK(dmi_get_stats(ring, &s) == DMI_OK);
    CHECK(s.launched_records == 12 && s.captured_records == 2 && s.dropped_records == 10);
    CHECK(s.captured_bytes == 2 * rb && s.dropped_bytes == 10 * rb && s.dropped_rows == 160);
    dmi_record_view_t v[4];
    uint32_t n = 0;
    CHECK(dmi_poll_host(ring, v, 4, &n) == DMI_OK && n == 2 && v[0].seq == 0 && v[1].seq == 1);
    CHECK(dmi_release_host(ring, 1) == DMI_OK);
    // first batch: points 1, 2 kept, then 3, 4, 3, 2 dropped; second batch: all of 1, 2, 3, 4, 3, 2 dropped
    const uint64_t want[5] = {0, 1, 3, 4, 2};
    for (uint32_t p = 0; p < 5; p++) {
        uint64_t d = 0;
        CHECK(dmi_get_point_drops(ring, p, &d) == DMI_OK && d == want[p]);
    }
    // room again: the next batch's first two are sequence numbers 12 and 13
    CHECK(dmi_observe_batch(ring, 6, points, datas, &src.t, &sel, &raw, 2, stream, &done) == DMI_OK && done == 6);
    CHECK(hipStreamSynchronize(stream) == hipSuccess);
    flush_all(ring);
    CHECK(dmi_poll_host(ring, v, 4, &n) == DMI_OK && n == 2 && v[0].seq == 12 && v[1].seq == 13);
    CHECK(dmi_ring_destroy(ring) == DMI_OK);
    CHECK(hipStreamDestroy(stream) == hipSuccess);
}

}  // namespace

int main(int argc, char **argv)
{
    const int n_iter = argc > 1 ? atoi(argv[1]) : 1500;
    fake_set_jitter_us(30);
    scenario("block, poll/release consumer, steps", DMI_POLICY_BLOCK, false, true, n_iter);
    scenario("drop-newest, poll/release consumer, steps", DMI_POLICY_DROP_NEWEST, false, true, n_iter);
    scenario("block, exporter as the consumer", DMI_POLICY_BLOCK, true, false, n_iter / 2);
    scenario("drop-newest, exporter as the consumer", DMI_POLICY_DROP_NEWEST, true, false, n_iter / 2);
    scenario_host_decided_drops();
    fprintf(stderr, "all scenarios passed\n");
    return 0;
}
