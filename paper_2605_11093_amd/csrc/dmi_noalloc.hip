// dmi_observe_into: one capture that allocates nothing, for callers that cannot call
// hipMalloc (code under HIP graph capture, tight serving loops, harnesses that forbid it).
//
// dmi_observe needs device memory beyond the observed tensor and the ring: the control block
// (head / tail copies, running counters, commit slot) and the request table staged for the
// kernel.  A ring allocates those when it is created.  Here they live in one file-scope device
// array, `scratch`, that exists once per GPU for as long as the process does; the record goes
// straight into memory of the caller's.  The capture kernels are the ones dmi_observe launches.
#include "dmi_ring.h"

using namespace dmi;
using namespace dmi::host;

namespace {

constexpr uint32_t kIntoMaxReqs = 1024;
// request table (4 words per request), first source row per request, and, for selections that
// take the decode-shaped kernel with several rows per request, the source row of every listed row
constexpr size_t kIntoTableWords = (size_t)kIntoMaxReqs * 5u + kDecodeMaxListed;

struct ScratchLayout {
    DevCtrl ctrl;
    alignas(16) uint32_t table[kIntoTableWords];
};

constexpr size_t kScratchBytes = 128u * 1024u;
static_assert(sizeof(ScratchLayout) <= kScratchBytes, "scratch layout outgrew the stated maximum");

}  // namespace

// The scratch memory: 128 KiB on every GPU the library runs on, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; what kernels and copies get
// is the per-device address kept in g_scratch_ptr below.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU, once looked up

// Address of this GPU's copy of `scratch` (every GPU holds its own, at its own address).
// `dev` is the calling thread's current device.
dmi_status_t scratch_on(int dev, ScratchLayout **out)
{
    if (dev < 0 || dev >= kMaxDevices) return fail(DMI_ERR_INVALID_ARG, "device ordinal %d is not supported", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(DMI_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<ScratchLayout *>(g_scratch_ptr[dev]);
    return DMI_OK;
}

}  // namespace

extern "C" dmi_status_t dmi_observe_into(uint32_t point_id, const dmi_tensor_t *t, const dmi_selection_t *sel,
                                         const dmi_transform_t *xf, uint64_t seq, uint64_t step_id,
                                         uint32_t rank_tag, void *out, uint64_t out_bytes,
                                         uint64_t *record_bytes, void *hip_stream)
{
    if (!t || !sel || !xf) return fail(DMI_ERR_INVALID_ARG, "tensor / selection / transform is NULL");
    if (point_id >= DMI_MAX_POINTS) return fail(DMI_ERR_INVALID_ARG, "point_id %u >= %u", point_id, DMI_MAX_POINTS);
    if (sel->n_reqs > kIntoMaxReqs)
        return fail(DMI_ERR_TOO_LARGE, "n_reqs %u is beyond the %u requests this entry point has scratch memory for",
                    sel->n_reqs, kIntoMaxReqs);
    if (sel->n_reqs && !sel->reqs) return fail(DMI_ERR_INVALID_ARG, "reqs is NULL");
    if (!transform_ok(t->dtype, xf->out_dtype))
        return fail(DMI_ERR_INVALID_ARG, "unsupported dtype pair %u -> %u", t->dtype, xf->out_dtype);
    if (xf->summary_mask & ~7u) return fail(DMI_ERR_INVALID_ARG, "bad summary_mask %u", xf->summary_mask);
    if (!out || (uintptr_t)out % 64u || out_bytes % 64u || out_bytes < DMI_HEADER_BYTES)
        return fail(DMI_ERR_INVALID_ARG, "out must be 64-byte aligned and out_bytes a multiple of 64");

    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    ScratchLayout *S = nullptr;
    dmi_status_t st = scratch_on(dev, &S);
    if (st != DMI_OK) return st;

    Geometry geo;
    CaptureArgs a;
    if ((st = prep_dense(t, sel, geo, a)) != DMI_OK) return st;
    uint64_t listed = 0;
    for (uint32_t i = 0; i < sel->n_reqs; i++) listed += sel->reqs[i].tok_count;
    const uint64_t ub = dmi_record_bytes(sel->n_reqs, listed, geo.row_elems, xf->out_dtype, xf->summary_mask);
    if (ub > out_bytes)
        return fail(DMI_ERR_TOO_LARGE, "the record may take %llu bytes, out_bytes is %llu", (unsigned long long)ub,
                    (unsigned long long)out_bytes);
    Plan pl;
    const PlanEnv env{static_cast<uint8_t *>(out), out_bytes, 0u, &S->ctrl, rank_tag, nullptr};
    if ((st = plan_capture(env, point_id, sel, xf, geo, a, pl, true)) != DMI_OK) return st;

    std::vector<uint32_t> words;
    selection_words(sel->reqs, sel->n_reqs, false, pl.row_map, words);
    if (words.size() > kIntoTableWords)
        return fail(DMI_ERR_TOO_LARGE, "the request table (%zu words) is beyond the scratch memory's %zu",
                    words.size(), kIntoTableWords);

    hipStream_t s = (hipStream_t)hip_stream;
    // the array keeps what the last call left: the stream starts at offset 0 with nothing counted
    HIP_TRY(launch_ctrl_reset(&S->ctrl, s));
    if (!words.empty()) HIP_TRY(launch_upload(S->table, words.data(), (uint32_t)words.size(), s));
    a.req_table = reinterpret_cast<const uint4 *>(S->table);
    a.row0 = S->table + 4u * (size_t)sel->n_reqs;
    a.row_map = pl.row_map ? a.row0 + sel->n_reqs : nullptr;
    a.seq = seq;
    a.step_id = step_id;
    a.cslot = &S->ctrl.slots[0];
    a.tail_floor = 0;
    a.drop_newest = 0;
    a.tail_src = nullptr;
    a.par_in = 0;
    a.step = nullptr;
    a.node = 0;
    a.n_batch = 1;
    BatchArgs b;
    memset(&b, 0, sizeof b);
    b.src[0] = a.src;
    b.point[0] = point_id;
    const hipError_t e = pl.decode ? launch_capture_decode(a, b, s) : launch_capture(a, b, pl.grid, geo.vec16, s);
    if (e != hipSuccess) return fail(DMI_ERR_HIP, "capture launch failed: %s", hipGetErrorString(e));
    if (record_bytes) *record_bytes = pl.ub;
    return DMI_OK;
}
