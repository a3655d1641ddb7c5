// The HookPoint operator dmi::observe(x, hook) as a native PyTorch operator (paper section 4.1:
// the hook is an ordinary operator of the framework, so that reaching it costs a dispatch and one
// launch, with no Python callback on the way, and a traced or compiled model carries it as a graph
// node).  This file is the front end only: it finds the arguments (the tensor's address, layout
// and current stream; the step's request selection) and calls the C ABI of dmi.h, which does the
// work.  It is built into a library of its own (libdmi_torch.so) so that libdmi.so stays free of
// any framework type.
//
// State lives in two small tables, addressed by integer handles that Python keeps:
//   step context   what every hook of a forward step shares (section 4.1, prepare_step): request
//                  selection, step id, keep vector; while a graph is being captured, the
//                  replayable step that collects the launches
//   hook           ring, point id, stored dtype, summary mask, its step context
#include <ATen/ATen.h>
#include <c10/hip/HIPStream.h>
#include <torch/library.h>

#include <cstdint>
#include <cstring>
#include <memory>
#include <mutex>
#include <shared_mutex>
#include <vector>

#include "dmi.h"

namespace {

struct StepCtx {
    std::vector<dmi_req_sel_t> reqs;
    bool has_reqs = false;
    uint64_t step_id = 0;
    const uint8_t *keep = nullptr;
    dmi_step_t *capturing = nullptr;        // non-null between capture begin and seal
    std::vector<uint32_t> nodes;            // records added to the step under capture
};

struct Hook {
    dmi_ring_t *ring = nullptr;
    uint32_t point = 0;
    int32_t out_dtype = -1;                 // -1: store the source dtype
    uint32_t summary_mask = 0;
    int32_t ctx = -1;
    bool live = false;
};

// Hooks fire from whichever threads run forward passes; the tables change only when models are
// built or torn down.  Entries are never moved once made (unique_ptr), so a reader needs the
// lock only to find its entry.  An entry's contents have no lock: a step context belongs to the
// thread that drives its model (it sets the step, then runs the forward whose hooks read it), as
// a ring belongs to one producer thread.
std::shared_mutex g_mu;
std::vector<std::unique_ptr<StepCtx>> g_ctx;
std::vector<std::unique_ptr<Hook>> g_hooks;

StepCtx *find_ctx(int32_t id)
{
    std::shared_lock<std::shared_mutex> lk(g_mu);
    return id >= 0 && (size_t)id < g_ctx.size() ? g_ctx[(size_t)id].get() : nullptr;
}

uint32_t dtype_code(const at::Tensor &x)
{
    switch (x.scalar_type()) {
    case at::kBFloat16: return DMI_DTYPE_BF16;
    case at::kHalf: return DMI_DTYPE_FP16;
    case at::kFloat: return DMI_DTYPE_FP32;
    default: TORCH_CHECK(false, "dmi::observe: unsupported dtype ", x.scalar_type());
    }
}

// x as [tokens, features] without a copy: the last dimension contiguous, all leading dimensions
// collapsible into one (each stride = the next inner one's stride times its size).
void rows_view(const at::Tensor &x, dmi_tensor_t &t)
{
    const int64_t nd = x.dim();
    TORCH_CHECK(nd >= 1, "dmi::observe: a HookPoint needs at least one dimension");
    const auto sz = x.sizes();
    const auto st = x.strides();
    TORCH_CHECK(st[nd - 1] == 1 || sz[nd - 1] <= 1,
                "dmi::observe: HookPoint needs a tensor whose rows are contiguous in memory");
    int64_t rows = 1, row_stride = 0;
    for (int64_t i = nd - 2; i >= 0; i--) {
        if (sz[i] == 1) continue;       // a dimension of one entry has no say
        if (!row_stride) row_stride = st[i];
        else TORCH_CHECK(rows == 0 || st[i] == row_stride * rows,
                         "dmi::observe: HookPoint needs a tensor whose rows are evenly spaced in memory");
        rows *= sz[i];
    }
    if (!row_stride) row_stride = sz[nd - 1];
    t.data = x.data_ptr();
    t.dtype = dtype_code(x);
    t.shape[0] = rows;
    t.shape[1] = sz[nd - 1];
    t.stride[0] = row_stride;
    t.stride[1] = 1;
}

void observe(at::Tensor &x, int64_t hook_id)
{
    Hook *h;
    {
        std::shared_lock<std::shared_mutex> lk(g_mu);
        TORCH_CHECK(hook_id >= 0 && (size_t)hook_id < g_hooks.size() && g_hooks[(size_t)hook_id]->live,
                    "dmi::observe: unknown hook ", hook_id);
        h = g_hooks[(size_t)hook_id].get();
    }
    StepCtx *c = find_ctx(h->ctx);
    TORCH_CHECK(c, "dmi::observe: hook ", hook_id, " has no step context");
    if (!c->has_reqs) return;           // no step prepared: the model runs unobserved
    dmi_tensor_t t;
    rows_view(x, t);
    dmi_selection_t sel;
    sel.n_reqs = (uint32_t)c->reqs.size();
    sel.reqs = c->reqs.data();
    sel.keep_mask_dev = c->keep;
    sel.row_index_dev = nullptr;
    dmi_transform_t xf;
    xf.out_dtype = h->out_dtype < 0 ? t.dtype : (uint32_t)h->out_dtype;
    xf.summary_mask = h->summary_mask;
    void *stream = c10::hip::getCurrentHIPStream(x.device().index()).stream();
    dmi_status_t st;
    if (c->capturing) {
        uint32_t node = 0;
        st = dmi_step_observe(c->capturing, h->point, &t, &sel, &xf, stream, &node);
        if (st == DMI_OK) c->nodes.push_back(node);
    } else {
        st = dmi_observe(h->ring, h->point, &t, &sel, &xf, c->step_id, stream);
    }
    TORCH_CHECK(st >= 0, "dmi::observe: status ", st, ": ", dmi_last_error());
}

}  // namespace

TORCH_LIBRARY(dmi, m)
{
    // Declared as writing x (it writes nothing): a call whose result nobody uses is then neither
    // dropped nor moved across other uses of the tensor by a compiler.
    m.def("observe(Tensor(a!) x, int hook) -> ()");
}

TORCH_LIBRARY_IMPL(dmi, CUDA, m)
{
    m.impl("observe", &observe);
}

extern "C" {

int32_t dmi_torch_ctx_create(void)
{
    std::unique_lock<std::shared_mutex> lk(g_mu);
    g_ctx.emplace_back(new StepCtx);
    return (int32_t)g_ctx.size() - 1;
}

// reqs [host] n entries of dmi_req_sel_t, copied; reqs == NULL: no step prepared (hooks launch nothing).
int32_t dmi_torch_ctx_set(int32_t ctx, uint64_t step_id, const dmi_req_sel_t *reqs, uint32_t n, const void *keep_mask_dev)
{
    StepCtx *c = find_ctx(ctx);
    if (!c) return DMI_ERR_INVALID_ARG;
    c->has_reqs = reqs != nullptr;
    if (reqs) c->reqs.assign(reqs, reqs + n); else c->reqs.clear();
    c->step_id = step_id;
    c->keep = static_cast<const uint8_t *>(keep_mask_dev);
    return DMI_OK;
}

// step != NULL: hooks add their launches to this replayable step (which must be open for capture)
// from now on; NULL: back to eager launches.  Starting a capture forgets the previous one's nodes.
int32_t dmi_torch_ctx_capture(int32_t ctx, dmi_step_t *step)
{
    StepCtx *c = find_ctx(ctx);
    if (!c) return DMI_ERR_INVALID_ARG;
    if (step) c->nodes.clear();
    c->capturing = step;
    return DMI_OK;
}

// Record indices of the launches added under the last capture; returns how many there are.
uint32_t dmi_torch_ctx_nodes(int32_t ctx, uint32_t *out, uint32_t max)
{
    StepCtx *c = find_ctx(ctx);
    if (!c) return 0;
    for (uint32_t i = 0; i < max && i < c->nodes.size(); i++) out[i] = c->nodes[i];
    return (uint32_t)c->nodes.size();
}

// out_dtype < 0: the record stores the source dtype.
int32_t dmi_torch_hook_create(dmi_ring_t *ring, uint32_t point_id, int32_t out_dtype, uint32_t summary_mask, int32_t ctx)
{
    if (!ring || !find_ctx(ctx)) return DMI_ERR_INVALID_ARG;
    std::unique_lock<std::shared_mutex> lk(g_mu);
    g_hooks.emplace_back(new Hook{ring, point_id, out_dtype, summary_mask, ctx, true});
    return (int32_t)g_hooks.size() - 1;
}

// The hook's ring is about to go, or the module is: later calls of the operator with this id fail.
int32_t dmi_torch_hook_destroy(int32_t hook)
{
    std::unique_lock<std::shared_mutex> lk(g_mu);
    if (hook < 0 || (size_t)hook >= g_hooks.size()) return DMI_ERR_INVALID_ARG;
    g_hooks[(size_t)hook]->live = false;
    g_hooks[(size_t)hook]->ring = nullptr;
    return DMI_OK;
}

}  // extern "C"
