// CPU executor behind the library's kernel-launch seam -- TEST INFRASTRUCTURE ONLY.
//
// Takes the place of the device code (csrc/dmi_kernels.hip) in the sanitizer build of the host
// runtime.  Every launcher enqueues a task on the (stand-in) stream that does what the host
// runtime relies on from a capture launch: the chain of head / tail copies, the drop decision,
// counters, commit slot, and a record with a true header and request table at the right
// place in the ring.  The payload is a fill pattern: nothing is gathered, converted or
// summarised here (this shares nothing with the oracle, and proves nothing about the kernels).
#include "dmi_ring.h"

namespace dmi {

uint32_t capture_lds_bytes(uint32_t, bool, bool) { return 0; }

namespace {

void ring_put(uint8_t *ring, uint64_t cap, uint64_t pos, const void *src, uint64_t n)
{
    const uint8_t *s = static_cast<const uint8_t *>(src);
    pos %= cap;
    const uint64_t first = n < cap - pos ? n : cap - pos;
    memcpy(ring + pos, s, first);
    if (n > first) memcpy(ring, s + first, n - first);
}

void ring_fill(uint8_t *ring, uint64_t cap, uint64_t pos, uint8_t value, uint64_t n)
{
    pos %= cap;
    const uint64_t first = n < cap - pos ? n : cap - pos;
    memset(ring + pos, value, first);
    if (n > first) memset(ring, value, n - first);
}

uint64_t load_u64(const uint64_t *p) { return __atomic_load_n(p, __ATOMIC_ACQUIRE); }

void model_capture(const CaptureArgs &a, const BatchArgs &b)
{
    DevCtrl *c = a.ctrl;
    const uint32_t par = a.par_in;
    const uint64_t head0 = c->head[par], tail_for = c->tail_for[par];
    uint64_t seq = a.seq, step_id = a.step_id, floor = a.tail_floor;
    uint32_t flags = a.drop_newest ? kStepDropNewest : 0u;
    if (a.step) {
        seq = a.step->seq_base + a.node;
        step_id = a.step->step_id;
        floor = a.step->tail_floor;
        flags = a.step->flags;
    }
    const bool drop_newest = (flags & kStepDropNewest) != 0;
    const uint64_t tail = drop_newest && tail_for > floor ? tail_for : floor;
    const uint64_t tail_now = load_u64(a.tail_src ? a.tail_src : &c->tail);
    const uint64_t next_tail_for = tail_now > tail_for ? tail_now : tail_for;
    if (flags & kStepSkip) {
        c->head[par ^ 1u] = head0;
        c->tail_for[par ^ 1u] = next_tail_for;
        return;
    }
    // rows kept: the listed ones, or what the keep vector leaves
    std::vector<uint32_t> kept(a.n_reqs);
    uint64_t n_rows = 0;
    for (uint32_t r = 0; r < a.n_reqs; r++) {
        kept[r] = (!a.keep_mask || a.keep_mask[r]) ? a.req_table[r].w : 0u;
        n_rows += kept[r];
    }
    const uint64_t rb = dmi_record_bytes(a.n_reqs, n_rows, a.row_elems, a.out_dtype, a.summary_mask);
    const uint64_t nb = a.n_batch;
    uint64_t n_fit = nb;
    if (drop_newest) {
        const uint64_t used = head0 - tail;
        n_fit = used < a.cap ? (a.cap - used) / rb : 0u;
        if (n_fit > nb) n_fit = nb;
    }
    if (a.force_drop) n_fit = 0;
    for (uint64_t y = 0; y < nb; y++) {
        if (y >= n_fit) { __atomic_fetch_add(&c->point_drops[b.point[y] & 4095u], 1u, __ATOMIC_RELAXED); continue; }
        const uint64_t at = head0 + y * rb;
        ring_fill(a.ring, a.cap, at, (uint8_t)(0x40u + ((seq + y) & 0x3Fu)), rb);
        uint32_t h[16] = {0};
        const uint64_t sy = seq + y, payload = n_rows * a.row_elems * dtype_size(a.out_dtype);
        h[0] = DMI_MAGIC; h[1] = 1u | (DMI_HEADER_BYTES << 16);
        h[2] = (uint32_t)sy; h[3] = (uint32_t)(sy >> 32);
        h[4] = (uint32_t)step_id; h[5] = (uint32_t)(step_id >> 32);
        h[6] = b.point[y];
        h[7] = a.src_dtype | (a.out_dtype << 8) | (a.summary_mask << 16) | (a.rec_flags << 24);
        h[8] = a.n_reqs; h[9] = (uint32_t)n_rows; h[10] = a.row_elems; h[11] = a.rank_tag;
        h[12] = (uint32_t)rb; h[13] = (uint32_t)(rb >> 32);
        h[14] = (uint32_t)payload; h[15] = (uint32_t)(payload >> 32);
        ring_put(a.ring, a.cap, at, h, 64);
        ring_fill(a.ring, a.cap, at + 64, 0, pad64((uint64_t)a.n_reqs * 16u));
        for (uint32_t r = 0; r < a.n_reqs; r++) {
            const uint32_t e[4] = {a.req_table[r].x, a.req_table[r].y, a.req_table[r].z, kept[r]};
            ring_put(a.ring, a.cap, at + 64 + 16ull * r, e, 16);
        }
    }
    // records behind the launched ones that the host has already decided to drop: counted here
    for (uint32_t i = 0; i < a.n_tail_drop; i++)
        __atomic_fetch_add(&c->point_drops[b.point[nb + i] & 4095u], 1u, __ATOMIC_RELAXED);
    const uint64_t n_drop = nb - n_fit + a.n_tail_drop;
    c->dropped_records += n_drop; c->dropped_rows += n_drop * n_rows; c->dropped_bytes += n_drop * rb;
    c->captured_records += n_fit; c->captured_rows += n_fit * n_rows; c->captured_bytes += n_fit * rb;
    const uint64_t new_head = head0 + n_fit * rb, last = seq + nb + a.n_tail_drop - 1u;
    c->head[par ^ 1u] = new_head;
    c->tail_for[par ^ 1u] = next_tail_for;
    CommitSlot *s = a.step ? &c->slots[last % kCommitSlots] : a.cslot;
    s->head = new_head;
    s->captured_records = c->captured_records; s->captured_rows = c->captured_rows; s->captured_bytes = c->captured_bytes;
    s->dropped_records = c->dropped_records; s->dropped_rows = c->dropped_rows; s->dropped_bytes = c->dropped_bytes;
    s->seq_plus1 = last + 1u;
}

}  // namespace

hipError_t launch_capture(const CaptureArgs &a, const BatchArgs &b, uint32_t grid, bool, hipStream_t s)
{
    if (grid == 0 || grid > kMaxGrid || a.n_batch == 0 || a.n_batch > kMaxBatch) return hipErrorInvalidValue;
    const CaptureArgs ac = a;
    const BatchArgs bc = b;
    fake_enqueue(s, [ac, bc] { model_capture(ac, bc); });
    return hipSuccess;
}

hipError_t launch_capture_decode(const CaptureArgs &a, const BatchArgs &b, hipStream_t s)
{
    if (a.n_batch == 0 || a.n_batch > kMaxBatch) return hipErrorInvalidValue;
    const CaptureArgs ac = a;
    const BatchArgs bc = b;
    fake_enqueue(s, [ac, bc] { model_capture(ac, bc); });
    return hipSuccess;
}

hipError_t launch_upload(uint32_t *dst, const uint32_t *words, uint32_t n_words, hipStream_t s)
{
    std::vector<uint32_t> w(words, words + n_words);      // kernel arguments carry the data
    fake_enqueue(s, [dst, w] { memcpy(dst, w.data(), w.size() * 4u); });
    return hipSuccess;
}

hipError_t launch_step_begin(DevCtrl *ctrl, StepParams *step, StepParams v, uint32_t par_from, uint32_t par_to,
                             const uint64_t *host_tail, hipStream_t s)
{
    fake_enqueue(s, [=] {
        *step = v;
        if (host_tail) ctrl->tail = load_u64(host_tail);
        if (par_from != par_to) {
            ctrl->head[par_to] = ctrl->head[par_from];
            ctrl->tail_for[par_to] = ctrl->tail_for[par_from];
        }
    });
    return hipSuccess;
}

hipError_t launch_ctrl_reset(DevCtrl *ctrl, hipStream_t s)
{
    fake_enqueue(s, [ctrl] { memset(ctrl, 0, offsetof(DevCtrl, point_drops)); });
    return hipSuccess;
}

hipError_t launch_fetch_slot(const CommitSlot *src, CommitSlot *dst_host, hipStream_t s)
{
    fake_enqueue(s, [src, dst_host] { memcpy(dst_host, src, sizeof(CommitSlot)); });
    return hipSuccess;
}

hipError_t launch_drain_kernel(const uint8_t *ring, uint64_t cap, uint8_t *host_ring, uint64_t host_cap,
                               uint64_t from, uint64_t nbytes, uint32_t, hipStream_t s)
{
    fake_enqueue(s, [=] {
        for (uint64_t i = 0; i < nbytes; i += 64u)
            memcpy(host_ring + (from + i) % host_cap, ring + (from + i) % cap, 64);
    });
    return hipSuccess;
}

}  // namespace dmi
