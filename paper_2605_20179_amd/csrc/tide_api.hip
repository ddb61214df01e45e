// C-ABI of libtide: context, expert packing, placement, the per-step call sequence,
// interval statistics and the refresh with its side-stream host-to-device copies.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include <chrono>

#include "host_experts.h"
#include "host_pack.h"
#include "packed12.h"
#include "tide_internal.h"

using namespace tide;

static_assert(kHostGateUpGroup == kGateUpGroup && kHostDownGroup == kDownGroup,
              "the host packer, the host experts and the GEMM kernels agree on the packed layout");

// Workspace of tide_moe_step_noalloc: one array per GPU, held until the process ends.  In host code the name is
// only a handle for hipGetSymbolAddress; every use of the memory goes through the per-device pointer below.
constexpr size_t kScratchBytes = (size_t)TIDE_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

thread_local std::string g_create_error;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
hipError_t scratch_on_device(int device, unsigned char** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || ((uintptr_t)p & 255)) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

struct Layer {
    LayerTables t{};
    uint16_t* slots_owned = nullptr;     // capacity+1 blobs
    const uint8_t* host_blobs = nullptr;
    uint64_t host_stride = 0;
    const uint8_t* comp_blobs = nullptr;  // 12-bit form of the same blobs: the source of refresh copies (optional for bf16 slots)
    uint64_t comp_stride = 0;
    uint8_t* expert_p12 = nullptr;        // device, [E + 1], 12-bit slots only: LayerTables::expert_p12
    bool shared_set = false;
    bool placed = false;
    hipEvent_t copies_begin = nullptr, copies_done = nullptr;
    hipEvent_t select_done = nullptr;    // the plan of the last refresh is in pinned memory
    bool result_pending = false;         // tide_refresh_async: the plan has not been read by the host yet
    bool copies_pending = false;         // a step must wait on copies_done before its GEMMs
    bool copies_recorded = false;
    RefreshOut* plan = nullptr;          // pinned, device-visible
    // deferred refresh: staging blobs, the tables the selection wrote, the slots the staged blobs go to
    uint8_t* staging = nullptr;
    int32_t* pend_slot_of = nullptr;
    int32_t* pend_eis = nullptr;
    std::vector<int> pend_slots;
    bool deferred_pending = false;
};

}  // namespace

// What one step in flight needs beyond its layer: a workspace, the second stream its large work items run on, and the
// events that fork onto and join from that stream.  The context owns one set for its ordinary calls; a stack step
// (tide_moe_stack_step) runs consecutive layers on several such sets ("lanes"), each with a stream of its own.
struct StepRes {
    Workspace ws{};
    hipStream_t aux = nullptr;
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
};
struct Lane {
    StepRes res{};
    hipStream_t stream = nullptr;
    hipEvent_t done = nullptr;
    std::vector<void*> allocs;
};

struct tide_ctx {
    tide_config cfg{};
    Shape shape{};
    int device = 0;
    Workspace ws{};
    std::vector<void*> ws_allocs;
    std::vector<Layer> layers;
    hipStream_t side = nullptr;             // refresh copies
    hipStream_t aux = nullptr;              // large work items run here, beside the small ones
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
    hipEvent_t compute_mark = nullptr;
    int max_rows = 0, max_tasks = 0;
    unsigned char* scratch_dev = nullptr;   // this device's copy of the static scratch array (tide_moe_step_noalloc)
    std::vector<Lane> lanes;                // tide_moe_stack_step: made on first use
    hipEvent_t stack_begin = nullptr;
    Workspace last{};                       // workspace of the most recent step (tide_step_histogram, tide_read_work_items)
    std::string err;
    // optional per-kernel timing: every kernel launch of a step stamps a start and a stop event
    int profiling = 0;                      // 0 off, 1 every kernel of a step, 2 the expert GEMMs, 3 gate/up and the kernel before it
    std::vector<hipEvent_t> prof_pool;      // created on demand, reused
    size_t prof_used = 0;
    std::vector<std::pair<int, std::pair<hipEvent_t, hipEvent_t>>> prof_spans;   // (kernel id, begin, end)
    int64_t steps_issued = 0;
    // host-core execution of misses (tide_host_experts / tide_moe_apply_misses_host)
    HostPool* pool = nullptr;
    hipEvent_t listed_ev = nullptr;         // the last exported miss list and its token states are in host memory
    bool listed_valid = false;
    const void* listed_miss = nullptr;      // the buffers, the size and the stream of the step that export speaks for
    const void* listed_hidden = nullptr;
    hipStream_t listed_stream = nullptr;
    int listed_cap = 0, listed_tokens = 0;
    tide_miss* h_miss = nullptr;            // pinned: [max_tokens * k]
    int32_t* h_n_miss = nullptr;            // pinned: [1]
    uint16_t* h_hidden = nullptr;           // pinned: [max_tokens][d]
    float* h_rows = nullptr;                // pinned, read by the device in place: [max_tokens][d]
    int32_t* h_tokens = nullptr;            // pinned, read by the device in place: [max_tokens]
    uint8_t* h_mask = nullptr;              // pinned, read by the device in place: [E] experts the GPU takes over the link
    int copy_engine = TIDE_COPY_KERNEL;     // who moves a refresh's blobs: the copy kernel, or one DMA per blob
    int link_share = 0;                     // percent of a step's missed experts evaluated by the GPU over the host link
    float host_ms[3] = {0.f, 0.f, 0.f};     // last call: wait for the list, host compute, whole call
};

namespace {

StepRes own_res(const tide_ctx* ctx) {
    StepRes r;
    r.ws = ctx->ws;
    r.aux = ctx->aux;
    r.fork_ev = ctx->fork_ev;
    r.join_ev = ctx->join_ev;
    return r;
}

int fail(tide_ctx* ctx, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_create_error = buf;
    return code;
}

#define TIDE_HIP(ctx, call)                                                                          \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess) return fail(ctx, TIDE_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

hipEvent_t prof_event(tide_ctx* ctx) {
    if (ctx->prof_used == ctx->prof_pool.size()) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        ctx->prof_pool.push_back(e);
    }
    return ctx->prof_pool[ctx->prof_used++];
}

// Runs `launch(ev)`; when profiling, ev carries two events that the launch stamps with the
// dispatch's begin and end times.
template <typename F>
hipError_t timed(tide_ctx* ctx, int kernel_id, F&& launch) {
    LaunchEvents ev;
    const bool gemm = kernel_id == TIDE_K_GATE_UP || kernel_id == TIDE_K_DOWN || kernel_id == TIDE_K_GATE_UP_BIG || kernel_id == TIDE_K_DOWN_BIG;
    const bool gate_up_and_before = kernel_id == TIDE_K_GATE_UP || kernel_id == TIDE_K_GATE_UP_BIG || kernel_id == TIDE_K_TOPK ||
                                    kernel_id == TIDE_K_DISPATCH;
    if (!ctx->profiling || (ctx->profiling == 2 && !gemm) || (ctx->profiling == 3 && !gate_up_and_before)) return launch(ev);
    ev.start = prof_event(ctx);
    ev.stop = prof_event(ctx);
    if (!ev.start || !ev.stop) return hipErrorOutOfMemory;
    hipError_t rc = launch(ev);
    if (rc == hipSuccess) ctx->prof_spans.push_back({kernel_id, {ev.start, ev.stop}});
    return rc;
}

int check_cfg(const tide_config* c) {
    if (!c) return fail(nullptr, TIDE_E_INVAL, "config is null");
    if (c->d <= 0 || c->d % 64) return fail(nullptr, TIDE_E_INVAL, "d must be a positive multiple of 64");
    if (c->d_ff <= 0 || c->d_ff % 64) return fail(nullptr, TIDE_E_INVAL, "d_ff must be a positive multiple of 64");
    if (c->n_experts < 1 || c->n_experts > kMaxExperts) return fail(nullptr, TIDE_E_INVAL, "n_experts must be 1..%d", kMaxExperts);
    if (c->top_k < 1 || c->top_k > kMaxTopK || c->top_k > c->n_experts) return fail(nullptr, TIDE_E_INVAL, "top_k must be 1..min(E,%d)", kMaxTopK);
    if (c->n_shared < 0 || c->n_shared > 1) return fail(nullptr, TIDE_E_INVAL, "n_shared must be 0 or 1");
    if (c->n_layers < 1) return fail(nullptr, TIDE_E_INVAL, "n_layers must be >= 1");
    if (c->capacity < 1 || c->capacity > c->n_experts) return fail(nullptr, TIDE_E_RANGE, "capacity must be 1..E");
    if (c->max_tokens < 1 || c->max_tokens > kMaxTokens) return fail(nullptr, TIDE_E_RANGE, "max_tokens must be 1..%d", kMaxTokens);
    if (c->gating != TIDE_GATING_SOFTMAX && c->gating != TIDE_GATING_SIGMOID) return fail(nullptr, TIDE_E_INVAL, "bad gating");
    if (c->bias_mode < TIDE_BIAS_NONE || c->bias_mode > TIDE_BIAS_SELECT) return fail(nullptr, TIDE_E_INVAL, "bad bias_mode");
    if (c->resident_format != TIDE_RESIDENT_BF16 && c->resident_format != TIDE_RESIDENT_P12) return fail(nullptr, TIDE_E_INVAL, "bad resident_format");
    return TIDE_OK;
}

template <typename T>
int ws_alloc(tide_ctx* ctx, T** p, size_t count) {
    void* q = nullptr;
    hipError_t e = hipMalloc(&q, count * sizeof(T) + 256);
    if (e != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "hipMalloc(%zu bytes): %s", count * sizeof(T), hipGetErrorString(e));
    ctx->ws_allocs.push_back(q);
    *p = static_cast<T*>(q);
    return TIDE_OK;
}

int layer_ok(tide_ctx* ctx, int layer) {
    if (!ctx) return TIDE_E_INVAL;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, TIDE_E_INVAL, "layer %d outside 0..%d", layer, ctx->cfg.n_layers - 1);
    return TIDE_OK;
}

uint16_t* slot_ptr(tide_ctx* ctx, Layer& L, int slot) { return L.slots_owned + (int64_t)slot * ctx->shape.blob_elems; }

int common_step(tide_ctx* ctx, const StepRes& res, int layer, const void* hidden_dev, int n_tokens, const int32_t* idx,
                const float* w, float* out_dev, tide_miss* miss_dev, int miss_cap, int32_t* n_miss_dev,
                hipStream_t stream, bool split_done) {
    Layer& L = ctx->layers[layer];
    const Workspace& ws = res.ws;
    if (!split_done)
        TIDE_HIP(ctx, timed(ctx, TIDE_K_DISPATCH, [&](LaunchEvents ev) {
            return launch_dispatch(ctx->shape, L.t, ws, idx, w, n_tokens, miss_dev, miss_cap, n_miss_dev, stream, ev); }));
    const int max_tasks = max_small_tasks_for(ctx->shape, n_tokens);
    const int max_big = max_big_tasks_for(ctx->shape, n_tokens);
    const uint16_t* x = static_cast<const uint16_t*>(hidden_dev);
    // The second stream forks here, after the split.  With host workers its first kernel hands the miss list
    // and the token states it names to pinned host memory: the list is final long before the step's GEMMs
    // end, and the host cores can start on it at once.
    if (ctx->pool || max_big > 0) {
        TIDE_HIP(ctx, hipEventRecord(res.fork_ev, stream));
        TIDE_HIP(ctx, hipStreamWaitEvent(res.aux, res.fork_ev, 0));
    }
    if (ctx->pool) {
        const int cap = std::min(miss_cap, n_tokens * ctx->cfg.top_k);
        TIDE_HIP(ctx, launch_miss_export(miss_dev, cap, n_miss_dev, x, n_tokens, ctx->cfg.d, ctx->h_miss, ctx->h_n_miss,
                                         ctx->h_hidden, res.aux));
        TIDE_HIP(ctx, hipEventRecord(ctx->listed_ev, res.aux));
        // a step recorded into a HIP graph hands its list over at every replay, but the event above then belongs to
        // the graph: the host path must not wait on it, it queues a hand-over of its own instead
        hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
        TIDE_HIP(ctx, hipStreamIsCapturing(stream, &capturing));
        ctx->listed_valid = capturing == hipStreamCaptureStatusNone;
        ctx->listed_miss = miss_dev;
        ctx->listed_hidden = hidden_dev;
        ctx->listed_stream = stream;
        ctx->listed_cap = cap;
        ctx->listed_tokens = n_tokens;
    }
    if (L.copies_pending) {                  // the GEMMs of both streams wait for a refresh's copies; nothing before them does
        TIDE_HIP(ctx, hipStreamWaitEvent(stream, L.copies_done, 0));
        if (max_big > 0) TIDE_HIP(ctx, hipStreamWaitEvent(res.aux, L.copies_done, 0));
        L.copies_pending = false;
    }
    // Small and large work items touch disjoint rows: the large ones run on the second stream so that
    // the two kinds of kernels overlap on the chip (join before the combine).
    if (max_big > 0) {
        TIDE_HIP(ctx, launch_plan_big(ws, max_big, res.aux));
        TIDE_HIP(ctx, timed(ctx, TIDE_K_GATE_UP_BIG, [&](LaunchEvents ev) {
            return launch_expert_gemm_big(0, ctx->shape, L.t, ws, x, max_big, res.aux, ev); }));
        TIDE_HIP(ctx, timed(ctx, TIDE_K_DOWN_BIG, [&](LaunchEvents ev) {
            return launch_expert_gemm_big(1, ctx->shape, L.t, ws, x, max_big, res.aux, ev); }));
        TIDE_HIP(ctx, hipEventRecord(res.join_ev, res.aux));
    }
    TIDE_HIP(ctx, timed(ctx, TIDE_K_GATE_UP, [&](LaunchEvents ev) {
        return launch_expert_gemm(0, ctx->shape, L.t, ws, x, max_tasks, stream, ev); }));
    TIDE_HIP(ctx, timed(ctx, TIDE_K_DOWN, [&](LaunchEvents ev) {
        return launch_expert_gemm(1, ctx->shape, L.t, ws, x, max_tasks, stream, ev); }));
    if (max_big > 0) TIDE_HIP(ctx, hipStreamWaitEvent(stream, res.join_ev, 0));
    else if (ctx->pool) TIDE_HIP(ctx, hipStreamWaitEvent(stream, ctx->listed_ev, 0));    // the export read hidden_dev
    TIDE_HIP(ctx, timed(ctx, TIDE_K_COMBINE, [&](LaunchEvents ev) {
        return launch_combine(ctx->shape, ws, w, n_tokens, out_dev, stream, ev); }));
    ctx->steps_issued++;
    ctx->last = res.ws;
    return TIDE_OK;
}

int step_args_ok(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens, float* out_dev,
                 tide_miss* miss_dev, int miss_cap, int32_t* n_miss_dev) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (n_tokens < 0 || n_tokens > ctx->cfg.max_tokens) return fail(ctx, TIDE_E_RANGE, "n_tokens %d outside 0..max_tokens=%d", n_tokens, ctx->cfg.max_tokens);
    if (!n_miss_dev) return fail(ctx, TIDE_E_INVAL, "n_miss_dev is null");
    if (miss_cap < 0 || (miss_cap > 0 && !miss_dev)) return fail(ctx, TIDE_E_INVAL, "miss_dev is null with miss_cap > 0");
    if (n_tokens > 0 && (!hidden_dev || !out_dev)) return fail(ctx, TIDE_E_INVAL, "hidden_dev / out_dev is null");
    if (((uintptr_t)hidden_dev & 15) || ((uintptr_t)out_dev & 15)) return fail(ctx, TIDE_E_INVAL, "hidden_dev / out_dev must be 16-byte aligned");
    Layer& L = ctx->layers[layer];
    if (!L.placed) return fail(ctx, TIDE_E_STATE, "layer %d has no placement: call tide_set_resident first", layer);
    if (ctx->cfg.n_shared && !L.shared_set) return fail(ctx, TIDE_E_STATE, "layer %d: shared expert not set", layer);
    return TIDE_OK;
}

// The listed misses (of the experts the mask keeps) evaluated on the GPU and added to out_dev: the work items'
// "slots" are expert ids and their weights the experts' pinned host blobs, which the GEMM kernels read in
// place across the host link.
int device_miss_pass(tide_ctx* ctx, Layer& L, const void* hidden_dev, int n_tokens, const tide_miss* miss_dev, int miss_cap,
                     const int32_t* n_miss_dev, float* out_dev, hipStream_t stream, const uint8_t* expert_mask) {
    const uint16_t* x = static_cast<const uint16_t*>(hidden_dev);
    LayerTables host_view = L.t;
    host_view.slots = reinterpret_cast<const uint16_t*>(L.host_blobs);
    host_view.expert_p12 = nullptr;                      // the host's blobs are bf16
    Shape shape = ctx->shape;
    shape.blob_elems = (int64_t)(L.host_stride / 2);
    const int max_small = max_miss_small_tasks_for(ctx->shape, n_tokens);
    const int max_big = max_miss_big_tasks_for(ctx->shape, n_tokens);
    TIDE_HIP(ctx, launch_clear_i32(ctx->ws.miss_hist, ctx->cfg.n_experts, stream));
    TIDE_HIP(ctx, launch_miss_group(ctx->shape, ctx->ws, miss_dev, miss_cap, n_miss_dev, n_tokens, max_big, stream, expert_mask));
    TIDE_HIP(ctx, launch_expert_gemm(0, shape, host_view, ctx->ws, x, max_small, stream));
    if (max_big > 0) TIDE_HIP(ctx, launch_plan_big(ctx->ws, max_big, stream));
    if (max_big > 0) TIDE_HIP(ctx, launch_expert_gemm_big(0, shape, host_view, ctx->ws, x, max_big, stream));
    TIDE_HIP(ctx, launch_expert_gemm(1, shape, host_view, ctx->ws, x, max_small, stream));
    if (max_big > 0) TIDE_HIP(ctx, launch_expert_gemm_big(1, shape, host_view, ctx->ws, x, max_big, stream));
    TIDE_HIP(ctx, launch_miss_combine(ctx->shape, ctx->ws, n_tokens, out_dev, stream));
    return TIDE_OK;
}

}  // namespace

extern "C" {

const char* tide_last_error(const tide_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

uint64_t tide_expert_blob_bytes(const tide_config* cfg) {
    if (!cfg) return 0;
    return 3ull * (uint64_t)cfg->d * (uint64_t)cfg->d_ff * 2ull;
}

int tide_pack_expert(const tide_config* cfg, const uint16_t* wg, const uint16_t* wu, const uint16_t* wd, void* blob) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!wg || !wu || !wd || !blob) return fail(nullptr, TIDE_E_INVAL, "null matrix or blob");
    pack_expert_blob(cfg->d, cfg->d_ff, wg, wu, wd, static_cast<uint16_t*>(blob));
    return TIDE_OK;
}

int tide_create(const tide_config* cfg, tide_ctx** out) {
    if (!out) return fail(nullptr, TIDE_E_INVAL, "out is null");
    *out = nullptr;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev < 1)
        return fail(nullptr, TIDE_E_HIP, "no HIP device: %s", e == hipSuccess ? "device count is 0" : hipGetErrorString(e));
    tide_ctx* ctx = new (std::nothrow) tide_ctx();
    if (!ctx) return fail(nullptr, TIDE_E_NOMEM, "out of host memory");
    ctx->cfg = *cfg;
    Shape& s = ctx->shape;
    s.d = cfg->d; s.E = cfg->n_experts; s.k = cfg->top_k; s.I = cfg->d_ff; s.n_shared = cfg->n_shared;
    s.capacity = cfg->capacity; s.gating = cfg->gating; s.bias_mode = cfg->bias_mode;
    s.blob_elems = 3ll * cfg->d * cfg->d_ff;
    s.resident_p12 = cfg->resident_format == TIDE_RESIDENT_P12;
    s.big_rows = s.resident_p12 ? kRowsPerBigTaskP12 : kRowsPerBigTask;
    auto bail = [&](int code) { g_create_error = ctx->err; tide_destroy(ctx); return code; };
    if (hipGetDevice(&ctx->device) != hipSuccess) return bail(fail(ctx, TIDE_E_HIP, "hipGetDevice failed"));
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) return bail(fail(ctx, TIDE_E_HIP, "hipGetDeviceProperties failed"));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return bail(fail(ctx, TIDE_E_HIP, "device is %s; libtide is built for gfx950 only", prop.gcnArchName));
    s.n_cus = prop.multiProcessorCount;

    if (hipError_t se = scratch_on_device(ctx->device, &ctx->scratch_dev); se != hipSuccess)
        return bail(fail(ctx, TIDE_E_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(se)));

    const int64_t N = cfg->max_tokens, P = N * cfg->top_k;
    ctx->max_rows = (int)(P + (cfg->n_shared ? N : 0));
    ctx->max_tasks = std::max(max_small_tasks_for(s, cfg->max_tokens), max_miss_small_tasks_for(s, cfg->max_tokens));
    const int max_big = std::max(max_big_tasks_for(s, cfg->max_tokens), max_miss_big_tasks_for(s, cfg->max_tokens));
    Workspace& w = ctx->ws;
    if ((rc = ws_alloc(ctx, &w.logits, (int64_t)kMaxRouterSplits * N * ((s.E + 15) / 16 * 16))) || (rc = ws_alloc(ctx, &w.topk_idx, P)) ||
        (rc = ws_alloc(ctx, &w.topk_w, P)) || (rc = ws_alloc(ctx, &w.hist_step, s.E)) ||
        (rc = ws_alloc(ctx, &w.row_token, ctx->max_rows)) || (rc = ws_alloc(ctx, &w.pair_row, P)) ||
        (rc = ws_alloc(ctx, &w.slot_off, s.capacity + 2)) || (rc = ws_alloc(ctx, &w.tasks, ctx->max_tasks)) ||
        (rc = ws_alloc(ctx, &w.big_tasks, max_big + 1)) || (rc = ws_alloc(ctx, &w.n_tasks, 2)) ||
        (rc = ws_alloc(ctx, &w.big_order, max_big + 1)) || (rc = ws_alloc(ctx, &w.act, (int64_t)ctx->max_rows * s.I)) ||
        (rc = ws_alloc(ctx, &w.y, (int64_t)ctx->max_rows * s.d)) || (rc = ws_alloc(ctx, &w.counts_tmp, s.E)) ||
        (rc = ws_alloc(ctx, &w.counters, 4)) || (rc = ws_alloc(ctx, &w.m_idx, P)) || (rc = ws_alloc(ctx, &w.m_tok, P)) ||
        (rc = ws_alloc(ctx, &w.m_w, P)) || (rc = ws_alloc(ctx, &w.miss_hist, s.E)) || (rc = ws_alloc(ctx, &w.m_count, 1)))
        return bail(rc);
    if (hipMemset(w.n_tasks, 0, 2 * sizeof(int32_t)) != hipSuccess || hipMemset(w.counters, 0, 4 * sizeof(int64_t)) != hipSuccess)
        return bail(fail(ctx, TIDE_E_HIP, "hipMemset failed"));

    if (hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) != hipSuccess ||
        hipStreamCreateWithFlags(&ctx->aux, hipStreamNonBlocking) != hipSuccess)
        return bail(fail(ctx, TIDE_E_HIP, "stream creation failed"));
    if (hipEventCreateWithFlags(&ctx->compute_mark, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->fork_ev, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->join_ev, hipEventDisableTiming) != hipSuccess)
        return bail(fail(ctx, TIDE_E_HIP, "event creation failed"));

    ctx->layers.resize(cfg->n_layers);
    for (Layer& L : ctx->layers) {
        int32_t *hits, *slot_of, *eis;
        if ((rc = ws_alloc(ctx, &hits, s.E)) || (rc = ws_alloc(ctx, &slot_of, s.E)) || (rc = ws_alloc(ctx, &eis, s.capacity)))
            return bail(rc);
        if (hipMemset(hits, 0, s.E * 4) != hipSuccess || hipMemset(slot_of, 0xFF, s.E * 4) != hipSuccess ||
            hipMemset(eis, 0xFF, s.capacity * 4) != hipSuccess)
            return bail(fail(ctx, TIDE_E_HIP, "hipMemset failed"));
        if ((rc = ws_alloc(ctx, &L.slots_owned, (int64_t)(s.capacity + 1) * s.blob_elems))) return bail(rc);
        L.t.hits = hits; L.t.slot_of = slot_of; L.t.expert_in_slot = eis; L.t.slots = L.slots_owned;
        if (s.resident_p12) {
            // which experts are kept in the 12-bit form: none until tide_register_compressed / tide_set_shared say so
            if ((rc = ws_alloc(ctx, &L.expert_p12, s.E + 1))) return bail(rc);
            if (hipMemset(L.expert_p12, 0, s.E + 1) != hipSuccess) return bail(fail(ctx, TIDE_E_HIP, "hipMemset failed"));
            L.t.expert_p12 = L.expert_p12;
        }
        if (hipEventCreate(&L.copies_begin) != hipSuccess || hipEventCreate(&L.copies_done) != hipSuccess ||
            hipEventCreateWithFlags(&L.select_done, hipEventDisableTiming) != hipSuccess)
            return bail(fail(ctx, TIDE_E_HIP, "event"));
        void* plan = nullptr;
        if (hipHostMalloc(&plan, sizeof(RefreshOut), hipHostMallocDefault) != hipSuccess) return bail(fail(ctx, TIDE_E_NOMEM, "pinned plan buffer"));
        L.plan = static_cast<RefreshOut*>(plan);
        memset(L.plan, 0, sizeof(RefreshOut));
    }
    if (hipDeviceSynchronize() != hipSuccess) return bail(fail(ctx, TIDE_E_HIP, "synchronize after set-up failed"));
    ctx->last = ctx->ws;
    *out = ctx;
    return TIDE_OK;
}

int tide_destroy(tide_ctx* ctx) {
    if (!ctx) return TIDE_OK;
    (void)hipDeviceSynchronize();
    for (Layer& L : ctx->layers) {
        if (L.copies_begin) (void)hipEventDestroy(L.copies_begin);
        if (L.copies_done) (void)hipEventDestroy(L.copies_done);
        if (L.select_done) (void)hipEventDestroy(L.select_done);
        if (L.plan) (void)hipHostFree(L.plan);
        if (L.staging) (void)hipFree(L.staging);
        if (L.pend_slot_of) (void)hipFree(L.pend_slot_of);
    }
    for (Lane& ln : ctx->lanes) {
        if (ln.done) (void)hipEventDestroy(ln.done);
        if (ln.res.fork_ev) (void)hipEventDestroy(ln.res.fork_ev);
        if (ln.res.join_ev) (void)hipEventDestroy(ln.res.join_ev);
        if (ln.stream) (void)hipStreamDestroy(ln.stream);
        if (ln.res.aux) (void)hipStreamDestroy(ln.res.aux);
        for (void* q : ln.allocs) (void)hipFree(q);
    }
    if (ctx->stack_begin) (void)hipEventDestroy(ctx->stack_begin);
    host_pool_destroy(ctx->pool);
    if (ctx->listed_ev) (void)hipEventDestroy(ctx->listed_ev);
    for (void* q : {(void*)ctx->h_miss, (void*)ctx->h_n_miss, (void*)ctx->h_hidden, (void*)ctx->h_rows, (void*)ctx->h_tokens, (void*)ctx->h_mask})
        if (q) (void)hipHostFree(q);
    for (hipEvent_t e : ctx->prof_pool) (void)hipEventDestroy(e);
    if (ctx->compute_mark) (void)hipEventDestroy(ctx->compute_mark);
    if (ctx->fork_ev) (void)hipEventDestroy(ctx->fork_ev);
    if (ctx->join_ev) (void)hipEventDestroy(ctx->join_ev);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    if (ctx->aux) (void)hipStreamDestroy(ctx->aux);
    for (void* p : ctx->ws_allocs) (void)hipFree(p);
    delete ctx;
    return TIDE_OK;
}

namespace {
// What a cache slot receives for expert e, byte for byte: the bf16 blob, or -- when the slots keep the 12-bit form and
// the expert has one -- its compressed blob.
struct BlobSource {
    const uint8_t* ptr;
    uint64_t bytes;
};
BlobSource resident_source(const tide_ctx* ctx, const Layer& L, int e) {
    if (ctx->shape.resident_p12) {
        const uint8_t* comp = L.comp_blobs + (uint64_t)e * L.comp_stride;
        if (!reinterpret_cast<const P12Header*>(comp)->raw) return {comp, tide_compressed_blob_bytes(&ctx->cfg)};
    }
    return {L.host_blobs + (uint64_t)e * L.host_stride, tide_expert_blob_bytes(&ctx->cfg)};
}
}  // namespace

int tide_register_experts(tide_ctx* ctx, int layer, const void* host_blobs, uint64_t blob_stride) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!host_blobs) return fail(ctx, TIDE_E_INVAL, "host_blobs is null");
    if (blob_stride < tide_expert_blob_bytes(&ctx->cfg) || (blob_stride & 15) || ((uintptr_t)host_blobs & 15))
        return fail(ctx, TIDE_E_INVAL, "blob_stride must be >= blob bytes; base and stride 16-byte aligned");
    // the refresh's copy kernel and the miss pass read the blobs in place: the memory must be pinned and
    // mapped into the device's address space (pageable memory would fault a kernel)
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host_blobs) != hipSuccess || attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr) {
        (void)hipGetLastError();
        return fail(ctx, TIDE_E_INVAL, "host_blobs must be pinned host memory (hipHostMalloc, or a tensor made with pin_memory=True)");
    }
    ctx->layers[layer].host_blobs = static_cast<const uint8_t*>(host_blobs);
    ctx->layers[layer].host_stride = blob_stride;
    return TIDE_OK;
}

uint64_t tide_compressed_blob_bytes(const tide_config* cfg) {
    if (!cfg) return 0;
    return p12_layout(tide_expert_blob_bytes(cfg) / 1024).bytes;
}

int tide_compress_expert(const tide_config* cfg, const void* blob_host, void* comp_host) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!blob_host || !comp_host) return fail(nullptr, TIDE_E_INVAL, "null matrix or blob pointer");
    compress_expert_blob(cfg->d, cfg->d_ff, static_cast<const uint16_t*>(blob_host), static_cast<uint8_t*>(comp_host));
    return TIDE_OK;
}

int tide_decompress_expert(const tide_config* cfg, const void* comp_host, void* blob_host) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!blob_host || !comp_host) return fail(nullptr, TIDE_E_INVAL, "null blob pointer");
    if (!decompress_expert_blob(cfg->d, cfg->d_ff, static_cast<const uint8_t*>(comp_host), static_cast<uint16_t*>(blob_host)))
        return fail(nullptr, TIDE_E_INVAL, "not a compressed blob of this configuration, or one marked raw");
    return TIDE_OK;
}

int tide_register_compressed(tide_ctx* ctx, int layer, const void* comp_host_blobs, uint64_t comp_stride) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    Layer& L = ctx->layers[layer];
    if (!comp_host_blobs) {                               // back to the raw blobs
        if (ctx->shape.resident_p12) return fail(ctx, TIDE_E_STATE, "12-bit slots are filled from the compressed blobs: they cannot be unregistered");
        TIDE_HIP(ctx, hipDeviceSynchronize());
        L.comp_blobs = nullptr;
        return TIDE_OK;
    }
    if (!L.host_blobs) return fail(ctx, TIDE_E_STATE, "layer %d: register the raw blobs first (tide_register_experts)", layer);
    if (comp_stride < tide_compressed_blob_bytes(&ctx->cfg) || (comp_stride & 63) || ((uintptr_t)comp_host_blobs & 63))
        return fail(ctx, TIDE_E_INVAL, "comp_stride must be >= the compressed size; base and stride 64-byte aligned");
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, comp_host_blobs) != hipSuccess || attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr) {
        (void)hipGetLastError();
        return fail(ctx, TIDE_E_INVAL, "comp_host_blobs must be pinned host memory");
    }
    const uint32_t n_tiles = (uint32_t)(tide_expert_blob_bytes(&ctx->cfg) / 1024);
    for (int e = 0; e < ctx->cfg.n_experts; ++e) {
        const P12Header* h = reinterpret_cast<const P12Header*>(static_cast<const uint8_t*>(comp_host_blobs) + (uint64_t)e * comp_stride);
        if (h->magic != kP12Magic || h->n_tiles != n_tiles || h->raw > 1)
            return fail(ctx, TIDE_E_INVAL, "expert %d: not a compressed blob of this configuration (tide_compress_expert)", e);
    }
    TIDE_HIP(ctx, hipDeviceSynchronize());
    if (ctx->shape.resident_p12) {
        std::vector<uint8_t> flags(ctx->cfg.n_experts);
        for (int e = 0; e < ctx->cfg.n_experts; ++e)
            flags[e] = reinterpret_cast<const P12Header*>(static_cast<const uint8_t*>(comp_host_blobs) + (uint64_t)e * comp_stride)->raw ? 0 : 1;
        TIDE_HIP(ctx, hipMemcpy(L.expert_p12, flags.data(), flags.size(), hipMemcpyHostToDevice));
        // what the slots hold was copied from the blobs registered before: the layer needs a placement again
        L.placed = false;
        L.copies_pending = false;
        L.deferred_pending = false;
        L.pend_slots.clear();
    }
    L.comp_blobs = static_cast<const uint8_t*>(comp_host_blobs);
    L.comp_stride = comp_stride;
    return TIDE_OK;
}

int tide_set_shared(tide_ctx* ctx, int layer, const void* blob_host) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!ctx->cfg.n_shared) return fail(ctx, TIDE_E_STATE, "context was created with n_shared = 0");
    if (!blob_host) return fail(ctx, TIDE_E_INVAL, "blob_host is null");
    Layer& L = ctx->layers[layer];
    TIDE_HIP(ctx, hipDeviceSynchronize());
    const uint64_t bytes = tide_expert_blob_bytes(&ctx->cfg);
    const void* src = blob_host;
    uint64_t src_bytes = bytes;
    std::vector<uint8_t> comp;
    if (ctx->shape.resident_p12) {
        comp.resize(tide_compressed_blob_bytes(&ctx->cfg));
        compress_expert_blob(ctx->cfg.d, ctx->cfg.d_ff, static_cast<const uint16_t*>(blob_host), comp.data());
        // every token of a step reaches the shared expert: in a context of many tokens per step its work items are the
        // widest of the step, and those are faster over the bf16 blob
        const uint8_t is_p12 = (reinterpret_cast<const P12Header*>(comp.data())->raw || ctx->cfg.max_tokens > kSharedP12MaxTokens) ? 0 : 1;
        if (is_p12) {
            src = comp.data();
            src_bytes = comp.size();
        }
        TIDE_HIP(ctx, hipMemcpy(L.expert_p12 + ctx->cfg.n_experts, &is_p12, 1, hipMemcpyHostToDevice));
    }
    TIDE_HIP(ctx, hipMemcpy(slot_ptr(ctx, L, ctx->cfg.capacity), src, src_bytes, hipMemcpyHostToDevice));
    L.shared_set = true;
    return TIDE_OK;
}

int tide_set_resident(tide_ctx* ctx, int layer, const int32_t* experts, int n) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    const int C = ctx->cfg.capacity, E = ctx->cfg.n_experts;
    if (n < 0 || n > C) return fail(ctx, TIDE_E_RANGE, "n = %d outside 0..capacity", n);
    if (n > 0 && !experts) return fail(ctx, TIDE_E_INVAL, "experts is null");
    Layer& L = ctx->layers[layer];
    if (!L.host_blobs) return fail(ctx, TIDE_E_STATE, "layer %d: experts not registered", layer);
    if (ctx->shape.resident_p12 && !L.comp_blobs)
        return fail(ctx, TIDE_E_STATE, "layer %d: 12-bit slots need the compressed blobs (tide_register_compressed)", layer);
    std::vector<int32_t> slot_of(E, -1), eis(C, -1);
    for (int s = 0; s < n; ++s) {
        const int e = experts[s];
        if (e == -1) continue;
        if (e < 0 || e >= E) return fail(ctx, TIDE_E_RANGE, "expert id %d outside 0..E-1", e);
        if (slot_of[e] >= 0) return fail(ctx, TIDE_E_INVAL, "expert %d listed twice", e);
        slot_of[e] = s;
        eis[s] = e;
    }
    TIDE_HIP(ctx, hipDeviceSynchronize());
    for (int s = 0; s < C; ++s)
        if (eis[s] >= 0) {
            const BlobSource src = resident_source(ctx, L, eis[s]);
            TIDE_HIP(ctx, hipMemcpy(slot_ptr(ctx, L, s), src.ptr, src.bytes, hipMemcpyHostToDevice));
        }
    TIDE_HIP(ctx, hipMemcpy(L.t.slot_of, slot_of.data(), E * 4, hipMemcpyHostToDevice));
    TIDE_HIP(ctx, hipMemcpy(L.t.expert_in_slot, eis.data(), C * 4, hipMemcpyHostToDevice));
    L.placed = true;
    L.copies_pending = false;
    L.deferred_pending = false;          // a placement set by hand supersedes a refresh that was not committed
    L.pend_slots.clear();
    return TIDE_OK;
}

namespace {
// tide_moe_step on the workspace `ws` (the context's own, or one carved from the static scratch array).
int moe_step_on(tide_ctx* ctx, const StepRes& res, int layer, const void* hidden_dev, int n_tokens, const float* router_w_dev,
                const float* router_bias_dev, float* out_dev, tide_miss* miss_dev, int miss_cap, int32_t* n_miss_dev,
                int32_t* topk_idx_dev, float* topk_w_dev, hipStream_t stream) {
    if (n_tokens == 0) {
        TIDE_HIP(ctx, launch_clear_i32(n_miss_dev, 1, stream));
        return TIDE_OK;
    }
    if (!router_w_dev) return fail(ctx, TIDE_E_INVAL, "router_w_dev is null");
    if (ctx->cfg.bias_mode != TIDE_BIAS_NONE && !router_bias_dev) return fail(ctx, TIDE_E_INVAL, "router_bias_dev is null but bias_mode != NONE");
    if ((uintptr_t)router_w_dev & 15) return fail(ctx, TIDE_E_INVAL, "router_w_dev must be 16-byte aligned");
    Layer& L = ctx->layers[layer];
    const Workspace& ws = res.ws;
    const uint16_t* x = static_cast<const uint16_t*>(hidden_dev);
    TIDE_HIP(ctx, timed(ctx, TIDE_K_ROUTER, [&](LaunchEvents ev) {
        return launch_router_logits(ctx->shape, x, n_tokens, router_w_dev, ws.logits, ws.hist_step, stream, ev); }));
    const bool one_wg = routes_in_one_workgroup(ctx->shape, n_tokens);
    if (one_wg) {
        TIDE_HIP(ctx, timed(ctx, TIDE_K_TOPK, [&](LaunchEvents ev) {
            return launch_route_small(ctx->shape, L.t, ws, router_bias_dev, n_tokens, topk_idx_dev, topk_w_dev, miss_dev,
                                      miss_cap, n_miss_dev, stream, ev); }));
    } else {
        TIDE_HIP(ctx, timed(ctx, TIDE_K_TOPK, [&](LaunchEvents ev) {
            return launch_topk_gate(ctx->shape, ws.logits, router_bias_dev, n_tokens, ws.topk_idx, ws.topk_w,
                                    ws.hist_step, topk_idx_dev, topk_w_dev, stream, ev); }));
    }
    return common_step(ctx, res, layer, hidden_dev, n_tokens, ws.topk_idx, ws.topk_w, out_dev, miss_dev, miss_cap,
                       n_miss_dev, stream, one_wg);
}
}  // namespace

int tide_moe_step(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens, const float* router_w_dev,
                  const float* router_bias_dev, float* out_dev, tide_miss* miss_dev, int miss_cap,
                  int32_t* n_miss_dev, int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream) {
    int rc = step_args_ok(ctx, layer, hidden_dev, n_tokens, out_dev, miss_dev, miss_cap, n_miss_dev);
    if (rc) return rc;
    return moe_step_on(ctx, own_res(ctx), layer, hidden_dev, n_tokens, router_w_dev, router_bias_dev, out_dev, miss_dev, miss_cap,
                       n_miss_dev, topk_idx_dev, topk_w_dev, static_cast<hipStream_t>(hip_stream));
}

namespace {
// The per-step buffers of a step over n_tokens tokens laid out from `base` on (each piece 256-byte aligned, with the
// same 256 bytes of slack behind it that tide_create gives its allocations); returns the bytes taken.  With base ==
// nullptr only the size is computed.  What outlives a step -- the step histogram, the running totals -- stays with
// the context, as do the buffers only the miss passes use.
size_t carve_step_workspace(const Shape& s, int n_tokens, unsigned char* base, Workspace& w) {
    size_t at = 0;
    auto take = [&](auto** field, size_t count) {
        using T = std::remove_pointer_t<std::remove_pointer_t<decltype(field)>>;
        if (base) *field = reinterpret_cast<T*>(base + at);
        at += (count * sizeof(T) + 256 + 255) / 256 * 256;
    };
    const size_t N = (size_t)n_tokens, P = N * s.k, rows = P + (s.n_shared ? N : 0);
    const size_t max_big = (size_t)max_big_tasks_for(s, n_tokens);
    take(&w.logits, (size_t)kMaxRouterSplits * N * ((s.E + 15) / 16 * 16));
    take(&w.topk_idx, P);
    take(&w.topk_w, P);
    take(&w.row_token, rows);
    take(&w.pair_row, P);
    take(&w.slot_off, (size_t)s.capacity + 2);
    take(&w.tasks, (size_t)max_small_tasks_for(s, n_tokens));
    take(&w.big_tasks, max_big + 1);
    take(&w.n_tasks, 2);
    take(&w.big_order, max_big + 1);
    take(&w.act, rows * s.I);
    take(&w.y, rows * s.d);
    return at;
}
}  // namespace

uint64_t tide_noalloc_scratch_bytes(void) { return kScratchBytes; }

int tide_moe_step_noalloc(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens, const float* router_w_dev,
                          const float* router_bias_dev, float* out_dev, tide_miss* miss_dev, int miss_cap,
                          int32_t* n_miss_dev, int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream) {
    int rc = step_args_ok(ctx, layer, hidden_dev, n_tokens, out_dev, miss_dev, miss_cap, n_miss_dev);
    if (rc) return rc;
    if (ctx->profiling) return fail(ctx, TIDE_E_STATE, "tide_moe_step_noalloc does not run while tide_profile is on (stamped launches create events)");
    StepRes res = own_res(ctx);
    Workspace& ws = res.ws;
    const size_t need = carve_step_workspace(ctx->shape, n_tokens, nullptr, ws);
    if (need > kScratchBytes)
        return fail(ctx, TIDE_E_RANGE, "a step of %d tokens needs %zu bytes of workspace; the static scratch array holds %zu",
                    n_tokens, need, kScratchBytes);
    carve_step_workspace(ctx->shape, n_tokens, ctx->scratch_dev, ws);
    return moe_step_on(ctx, res, layer, hidden_dev, n_tokens, router_w_dev, router_bias_dev, out_dev, miss_dev, miss_cap,
                       n_miss_dev, topk_idx_dev, topk_w_dev, static_cast<hipStream_t>(hip_stream));
}

namespace {
constexpr int kStackLanes = 2;

// The lanes of tide_moe_stack_step: each a workspace of the context's size (the step histogram and the running totals
// excepted, which stay the context's), a stream, a second stream for large work items and their events.
int make_lanes(tide_ctx* ctx) {
    if (!ctx->lanes.empty()) return TIDE_OK;
    std::vector<Lane> lanes(kStackLanes);
    auto undo = [&](int code) {
        for (Lane& ln : lanes) {
            if (ln.done) (void)hipEventDestroy(ln.done);
            if (ln.res.fork_ev) (void)hipEventDestroy(ln.res.fork_ev);
            if (ln.res.join_ev) (void)hipEventDestroy(ln.res.join_ev);
            if (ln.stream) (void)hipStreamDestroy(ln.stream);
            if (ln.res.aux) (void)hipStreamDestroy(ln.res.aux);
            for (void* q : ln.allocs) (void)hipFree(q);
        }
        return code;
    };
    const size_t bytes = carve_step_workspace(ctx->shape, ctx->cfg.max_tokens, nullptr, lanes[0].res.ws) + (size_t)ctx->cfg.n_experts * 4 + 512;
    for (Lane& ln : lanes) {
        void* p = nullptr;
        if (hipMalloc(&p, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return undo(fail(ctx, TIDE_E_NOMEM, "out of device memory for a stack lane's workspace (%zu bytes)", bytes));
        }
        ln.allocs.push_back(p);
        ln.res.ws = ctx->ws;                       // counters and the miss-pass buffers stay the context's
        const size_t used = carve_step_workspace(ctx->shape, ctx->cfg.max_tokens, static_cast<unsigned char*>(p), ln.res.ws);
        ln.res.ws.hist_step = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(p) + used);
        if (hipStreamCreateWithFlags(&ln.stream, hipStreamNonBlocking) != hipSuccess ||
            hipStreamCreateWithFlags(&ln.res.aux, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&ln.done, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&ln.res.fork_ev, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&ln.res.join_ev, hipEventDisableTiming) != hipSuccess)
            return undo(fail(ctx, TIDE_E_HIP, "stream / event creation for a stack lane failed"));
    }
    if (!ctx->stack_begin && hipEventCreateWithFlags(&ctx->stack_begin, hipEventDisableTiming) != hipSuccess)
        return undo(fail(ctx, TIDE_E_HIP, "event creation failed"));
    ctx->lanes = std::move(lanes);
    return TIDE_OK;
}
}  // namespace

int tide_moe_stack_step(tide_ctx* ctx, int first_layer, int n_layers, const void* const* hidden_dev, int n_tokens,
                        const float* const* router_w_dev, const float* const* router_bias_dev, float* const* out_dev,
                        tide_miss* const* miss_dev, int miss_cap, int32_t* const* n_miss_dev, void* hip_stream) {
    if (!ctx) return TIDE_E_INVAL;
    if (n_layers < 0 || first_layer < 0 || first_layer + n_layers > ctx->cfg.n_layers)
        return fail(ctx, TIDE_E_INVAL, "layers %d..%d outside 0..%d", first_layer, first_layer + n_layers - 1, ctx->cfg.n_layers - 1);
    if (n_layers == 0) return TIDE_OK;
    if (!hidden_dev || !router_w_dev || !out_dev || !n_miss_dev || (miss_cap > 0 && !miss_dev))
        return fail(ctx, TIDE_E_INVAL, "null pointer array");
    if (ctx->cfg.bias_mode != TIDE_BIAS_NONE && !router_bias_dev) return fail(ctx, TIDE_E_INVAL, "router_bias_dev is null but bias_mode != NONE");
    if (ctx->pool) return fail(ctx, TIDE_E_STATE, "tide_moe_stack_step does not run with host workers (tide_host_experts): their hand-over buffers serve one step at a time");
    for (int i = 0; i < n_layers; ++i) {
        int rc = step_args_ok(ctx, first_layer + i, hidden_dev[i], n_tokens, out_dev[i], miss_cap > 0 ? miss_dev[i] : nullptr, miss_cap, n_miss_dev[i]);
        if (rc) return rc;
        if (n_tokens > 0 && !router_w_dev[i]) return fail(ctx, TIDE_E_INVAL, "router_w_dev[%d] is null", i);
    }
    int rc = make_lanes(ctx);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // every lane starts behind what the caller has queued, and the caller's stream continues behind every lane
    TIDE_HIP(ctx, hipEventRecord(ctx->stack_begin, stream));
    const int used = std::min(n_layers, (int)ctx->lanes.size());
    for (int j = 0; j < used; ++j) TIDE_HIP(ctx, hipStreamWaitEvent(ctx->lanes[j].stream, ctx->stack_begin, 0));
    for (int i = 0; i < n_layers; ++i) {
        Lane& ln = ctx->lanes[i % ctx->lanes.size()];
        rc = moe_step_on(ctx, ln.res, first_layer + i, hidden_dev[i], n_tokens, router_w_dev[i], router_bias_dev ? router_bias_dev[i] : nullptr,
                         out_dev[i], miss_cap > 0 ? miss_dev[i] : nullptr, miss_cap, n_miss_dev[i], nullptr, nullptr, ln.stream);
        if (rc) break;
    }
    for (int j = 0; j < used; ++j) {
        TIDE_HIP(ctx, hipEventRecord(ctx->lanes[j].done, ctx->lanes[j].stream));
        TIDE_HIP(ctx, hipStreamWaitEvent(stream, ctx->lanes[j].done, 0));
    }
    return rc;
}

int tide_moe_step_routed(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens, const int32_t* topk_idx_dev,
                         const float* topk_w_dev, float* out_dev, tide_miss* miss_dev, int miss_cap,
                         int32_t* n_miss_dev, void* hip_stream) {
    int rc = step_args_ok(ctx, layer, hidden_dev, n_tokens, out_dev, miss_dev, miss_cap, n_miss_dev);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (n_tokens == 0) {
        TIDE_HIP(ctx, launch_clear_i32(n_miss_dev, 1, stream));
        return TIDE_OK;
    }
    if (!topk_idx_dev || !topk_w_dev) return fail(ctx, TIDE_E_INVAL, "topk_idx_dev / topk_w_dev is null");
    if ((uintptr_t)topk_idx_dev & 15) return fail(ctx, TIDE_E_INVAL, "topk_idx_dev must be 16-byte aligned");
    TIDE_HIP(ctx, launch_count_pairs(ctx->shape, topk_idx_dev, n_tokens, ctx->ws.hist_step, stream));
    return common_step(ctx, own_res(ctx), layer, hidden_dev, n_tokens, topk_idx_dev, topk_w_dev, out_dev, miss_dev, miss_cap,
                       n_miss_dev, stream, false);
}

int tide_moe_apply_misses(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens, const tide_miss* miss_dev,
                          int miss_cap, const int32_t* n_miss_dev, float* out_dev, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (n_tokens < 0 || n_tokens > ctx->cfg.max_tokens) return fail(ctx, TIDE_E_RANGE, "n_tokens %d outside 0..max_tokens=%d", n_tokens, ctx->cfg.max_tokens);
    if (n_tokens == 0 || miss_cap == 0) return TIDE_OK;
    if (!hidden_dev || !out_dev || !miss_dev || !n_miss_dev) return fail(ctx, TIDE_E_INVAL, "null argument");
    if (miss_cap < 0 || (int64_t)miss_cap > (int64_t)ctx->cfg.max_tokens * ctx->cfg.top_k) return fail(ctx, TIDE_E_RANGE, "miss_cap outside 0..max_tokens*k");
    if (((uintptr_t)hidden_dev & 15) || ((uintptr_t)out_dev & 15)) return fail(ctx, TIDE_E_INVAL, "hidden_dev / out_dev must be 16-byte aligned");
    Layer& L = ctx->layers[layer];
    if (!L.host_blobs) return fail(ctx, TIDE_E_STATE, "layer %d: experts not registered", layer);
    return device_miss_pass(ctx, L, hidden_dev, n_tokens, miss_dev, miss_cap, n_miss_dev, out_dev,
                            static_cast<hipStream_t>(hip_stream), nullptr);
}

int tide_host_experts(tide_ctx* ctx, int n_threads) {
    if (!ctx) return TIDE_E_INVAL;
    if (n_threads < 0 || n_threads > 1024) return fail(ctx, TIDE_E_RANGE, "n_threads must be 0..1024");
    TIDE_HIP(ctx, hipDeviceSynchronize());
    host_pool_destroy(ctx->pool);
    ctx->pool = nullptr;
    ctx->listed_valid = false;
    if (n_threads == 0) return TIDE_OK;
    if (!ctx->h_tokens) {
        const size_t N = ctx->cfg.max_tokens, P = N * ctx->cfg.top_k, d = ctx->cfg.d;
        if (!ctx->listed_ev) TIDE_HIP(ctx, hipEventCreateWithFlags(&ctx->listed_ev, hipEventDisableTiming));
        for (void* old : {(void*)ctx->h_miss, (void*)ctx->h_n_miss, (void*)ctx->h_hidden, (void*)ctx->h_rows, (void*)ctx->h_mask})
            if (old) (void)hipHostFree(old);
        ctx->h_miss = nullptr; ctx->h_n_miss = nullptr; ctx->h_hidden = nullptr; ctx->h_rows = nullptr; ctx->h_mask = nullptr;
        void* q = nullptr;
        if (hipHostMalloc(&q, P * sizeof(tide_miss), hipHostMallocDefault) != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "pinned miss list");
        ctx->h_miss = static_cast<tide_miss*>(q);
        if (hipHostMalloc(&q, 64, hipHostMallocDefault) != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "pinned counter");
        ctx->h_n_miss = static_cast<int32_t*>(q);
        if (hipHostMalloc(&q, N * d * 2, hipHostMallocDefault) != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "pinned token states");
        ctx->h_hidden = static_cast<uint16_t*>(q);
        if (hipHostMalloc(&q, N * d * 4, hipHostMallocDefault) != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "pinned result rows");
        ctx->h_rows = static_cast<float*>(q);
        if (hipHostMalloc(&q, (size_t)ctx->cfg.n_experts + 64, hipHostMallocDefault) != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "pinned expert mask");
        ctx->h_mask = static_cast<uint8_t*>(q);
        if (hipHostMalloc(&q, N * 4, hipHostMallocDefault) != hipSuccess) return fail(ctx, TIDE_E_NOMEM, "pinned row tokens");
        ctx->h_tokens = static_cast<int32_t*>(q);
    }
    ctx->pool = host_pool_create(n_threads);
    return TIDE_OK;
}

int tide_moe_apply_misses_host(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens, const tide_miss* miss_dev,
                               int miss_cap, const int32_t* n_miss_dev, float* out_dev, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!ctx->pool) return fail(ctx, TIDE_E_STATE, "no host workers: call tide_host_experts first");
    if (n_tokens < 0 || n_tokens > ctx->cfg.max_tokens) return fail(ctx, TIDE_E_RANGE, "n_tokens %d outside 0..max_tokens=%d", n_tokens, ctx->cfg.max_tokens);
    if (n_tokens == 0 || miss_cap == 0) return TIDE_OK;
    if (!hidden_dev || !out_dev || !miss_dev || !n_miss_dev) return fail(ctx, TIDE_E_INVAL, "null argument");
    if (miss_cap < 0 || (int64_t)miss_cap > (int64_t)ctx->cfg.max_tokens * ctx->cfg.top_k) return fail(ctx, TIDE_E_RANGE, "miss_cap outside 0..max_tokens*k");
    if (((uintptr_t)hidden_dev & 15) || ((uintptr_t)out_dev & 15)) return fail(ctx, TIDE_E_INVAL, "hidden_dev / out_dev must be 16-byte aligned");
    Layer& L = ctx->layers[layer];
    if (!L.host_blobs) return fail(ctx, TIDE_E_STATE, "layer %d: experts not registered", layer);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const auto t0 = std::chrono::steady_clock::now();
    // The list and the token states reach the host through a kernel on the second stream.  If they are the buffers
    // of the last step issued on this stream, that step has queued the export right behind its split, so the host
    // cores work while the GPU is still on the step's expert GEMMs; otherwise the export is queued now, behind all
    // work on hip_stream.
    const int cap = std::min(miss_cap, n_tokens * ctx->cfg.top_k);
    if (!(ctx->listed_valid && ctx->listed_miss == miss_dev && ctx->listed_hidden == hidden_dev && ctx->listed_stream == stream &&
          ctx->listed_cap == cap && ctx->listed_tokens == n_tokens)) {
        TIDE_HIP(ctx, hipEventRecord(ctx->fork_ev, stream));
        TIDE_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->fork_ev, 0));
        TIDE_HIP(ctx, launch_miss_export(miss_dev, cap, n_miss_dev, static_cast<const uint16_t*>(hidden_dev), n_tokens, ctx->cfg.d,
                                         ctx->h_miss, ctx->h_n_miss, ctx->h_hidden, ctx->aux));
        TIDE_HIP(ctx, hipEventRecord(ctx->listed_ev, ctx->aux));
    }
    ctx->listed_valid = false;
    TIDE_HIP(ctx, hipEventSynchronize(ctx->listed_ev));
    const auto t1 = std::chrono::steady_clock::now();
    const int n = std::max(0, std::min(*ctx->h_n_miss, cap));
    const int E = ctx->cfg.n_experts;
    for (int i = 0; i < n; ++i)
        if (ctx->h_miss[i].token < 0 || ctx->h_miss[i].token >= n_tokens || ctx->h_miss[i].expert < 0 || ctx->h_miss[i].expert >= E)
            return fail(ctx, TIDE_E_INVAL, "the miss list names a token or an expert out of range");
    // Optionally the GPU takes a share of the missed experts -- those with the most tokens -- and evaluates them
    // over the host link, queued behind the step on hip_stream, while the host workers do the rest.
    const uint8_t* skip = nullptr;
    if (ctx->link_share > 0 && n > 0) {
        std::vector<int32_t> cnt(E, 0), order;
        for (int i = 0; i < n; ++i) cnt[ctx->h_miss[i].expert]++;
        for (int e = 0; e < E; ++e)
            if (cnt[e]) order.push_back(e);
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cnt[a] > cnt[b]; });
        const int take = (int)((int64_t)order.size() * ctx->link_share / 100);
        if (take > 0) {
            memset(ctx->h_mask, 0, E);
            for (int j = 0; j < take; ++j) ctx->h_mask[order[j]] = 1;
            skip = ctx->h_mask;
            rc = device_miss_pass(ctx, L, hidden_dev, n_tokens, miss_dev, cap, n_miss_dev, out_dev, stream, ctx->h_mask);
            if (rc) return rc;
        }
    }
    const int rows = host_apply_misses(ctx->pool, L.host_blobs, L.host_stride, ctx->cfg.d, ctx->cfg.d_ff, E,
                                       ctx->h_hidden, n_tokens, ctx->h_miss, n, ctx->h_rows, ctx->h_tokens, skip);
    const auto t2 = std::chrono::steady_clock::now();
    if (rows < 0) return fail(ctx, TIDE_E_INVAL, "the miss list names a token or an expert out of range");
    // the rows are added by a kernel that reads them in place from pinned host memory, after the step's own combine
    TIDE_HIP(ctx, launch_add_rows(ctx->h_rows, ctx->h_tokens, rows, ctx->cfg.d, out_dev, stream));
    const auto t3 = std::chrono::steady_clock::now();
    auto ms = [](auto a, auto b) { return std::chrono::duration<float, std::milli>(b - a).count(); };
    ctx->host_ms[0] = ms(t0, t1);
    ctx->host_ms[1] = ms(t1, t2);
    ctx->host_ms[2] = ms(t0, t3);
    return TIDE_OK;
}

int tide_host_link_share(tide_ctx* ctx, int percent) {
    if (!ctx) return TIDE_E_INVAL;
    if (percent < 0 || percent > 100) return fail(ctx, TIDE_E_RANGE, "percent must be 0..100");
    ctx->link_share = percent;
    return TIDE_OK;
}

int tide_host_miss_ms(tide_ctx* ctx, float* ms3_host) {
    if (!ctx) return TIDE_E_INVAL;
    if (!ms3_host) return fail(ctx, TIDE_E_INVAL, "ms3_host is null");
    memcpy(ms3_host, ctx->host_ms, sizeof ctx->host_ms);
    return TIDE_OK;
}

int tide_host_misses(const tide_config* cfg, const void* blobs_host, uint64_t blob_stride, const uint16_t* x_host, int n_tokens,
                     const tide_miss* miss_host, int n_miss, int n_threads, float* out_host) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (n_tokens < 0 || n_tokens > cfg->max_tokens) return fail(nullptr, TIDE_E_RANGE, "n_tokens outside 0..max_tokens");
    if (n_miss < 0 || (int64_t)n_miss > (int64_t)n_tokens * cfg->top_k) return fail(nullptr, TIDE_E_RANGE, "n_miss outside 0..n_tokens*k");
    if (n_threads < 1 || n_threads > 1024) return fail(nullptr, TIDE_E_RANGE, "n_threads must be 1..1024");
    if (n_miss == 0) return TIDE_OK;
    if (!blobs_host || !x_host || !miss_host || !out_host) return fail(nullptr, TIDE_E_INVAL, "null argument");
    if (blob_stride < tide_expert_blob_bytes(cfg) || (blob_stride & 15)) return fail(nullptr, TIDE_E_INVAL, "blob_stride must be >= blob bytes and 16-byte aligned");
    std::vector<float> rows((size_t)std::min(n_miss, n_tokens) * cfg->d);
    std::vector<int32_t> tokens(std::min(n_miss, n_tokens));
    HostPool* pool = host_pool_create(n_threads);
    const int n_rows = host_apply_misses(pool, static_cast<const uint8_t*>(blobs_host), blob_stride, cfg->d, cfg->d_ff, cfg->n_experts,
                                         x_host, n_tokens, miss_host, n_miss, rows.data(), tokens.data());
    host_pool_destroy(pool);
    if (n_rows < 0) return fail(nullptr, TIDE_E_INVAL, "the miss list names a token or an expert out of range");
    for (int r = 0; r < n_rows; ++r) {
        float* o = out_host + (int64_t)tokens[r] * cfg->d;
        const float* v = rows.data() + (int64_t)r * cfg->d;
        for (int c = 0; c < cfg->d; ++c) o[c] += v[c];
    }
    return TIDE_OK;
}

int tide_host_expert(const tide_config* cfg, const void* blob_host, const uint16_t* x_host, int m, float* y_host) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (m < 0) return fail(nullptr, TIDE_E_RANGE, "m is negative");
    if (m == 0) return TIDE_OK;
    if (!blob_host || !x_host || !y_host) return fail(nullptr, TIDE_E_INVAL, "null argument");
    host_expert_forward(blob_host, cfg->d, cfg->d_ff, x_host, m, y_host);
    return TIDE_OK;
}

int tide_interval_stats(tide_ctx* ctx, int layer, int32_t* counts_host, int reset, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!counts_host) return fail(ctx, TIDE_E_INVAL, "counts_host is null");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    Layer& L = ctx->layers[layer];
    TIDE_HIP(ctx, hipMemcpyAsync(counts_host, L.t.hits, ctx->cfg.n_experts * 4, hipMemcpyDeviceToHost, stream));
    if (reset) TIDE_HIP(ctx, launch_clear_i32(L.t.hits, ctx->cfg.n_experts, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    return TIDE_OK;
}

int tide_set_counts(tide_ctx* ctx, int layer, const int32_t* counts_host, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!counts_host) return fail(ctx, TIDE_E_INVAL, "counts_host is null");
    for (int e = 0; e < ctx->cfg.n_experts; ++e)
        if (counts_host[e] < 0) return fail(ctx, TIDE_E_RANGE, "counts_host[%d] is negative", e);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TIDE_HIP(ctx, hipMemcpyAsync(ctx->layers[layer].t.hits, counts_host, (size_t)ctx->cfg.n_experts * 4, hipMemcpyHostToDevice, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    return TIDE_OK;
}

int tide_read_work_items(tide_ctx* ctx, tide_work_item* items_host, int items_cap, int* n_items_host, int32_t* row_token_host,
                         int rows_cap, int* n_rows_host, void* hip_stream) {
    if (!ctx) return TIDE_E_INVAL;
    if (!n_items_host || !n_rows_host || items_cap < 0 || rows_cap < 0 || (items_cap > 0 && !items_host) || (rows_cap > 0 && !row_token_host))
        return fail(ctx, TIDE_E_INVAL, "null output");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int32_t n_tasks[2] = {0, 0}, total_rows = 0;
    TIDE_HIP(ctx, hipMemcpyAsync(n_tasks, ctx->last.n_tasks, sizeof n_tasks, hipMemcpyDeviceToHost, stream));
    TIDE_HIP(ctx, hipMemcpyAsync(&total_rows, ctx->last.slot_off + ctx->cfg.capacity + 1, sizeof total_rows, hipMemcpyDeviceToHost, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    if (ctx->steps_issued == 0) n_tasks[0] = n_tasks[1] = total_rows = 0;
    std::vector<Task> small((size_t)std::max(n_tasks[0], 0)), big((size_t)std::max(n_tasks[1], 0));
    if (!small.empty()) TIDE_HIP(ctx, hipMemcpyAsync(small.data(), ctx->last.tasks, small.size() * sizeof(Task), hipMemcpyDeviceToHost, stream));
    if (!big.empty()) TIDE_HIP(ctx, hipMemcpyAsync(big.data(), ctx->last.big_tasks, big.size() * sizeof(Task), hipMemcpyDeviceToHost, stream));
    const int n_rows = std::min(std::max(total_rows, 0), ctx->max_rows);
    if (std::min(n_rows, rows_cap) > 0)
        TIDE_HIP(ctx, hipMemcpyAsync(row_token_host, ctx->last.row_token, (size_t)std::min(n_rows, rows_cap) * 4, hipMemcpyDeviceToHost, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    int at = 0;
    for (int kind = 0; kind < 2; ++kind)
        for (const Task& t : (kind ? big : small)) {
            if (at < items_cap) items_host[at] = tide_work_item{t.slot, t.row0, t.nrows, kind};
            ++at;
        }
    *n_items_host = at;
    *n_rows_host = n_rows;
    return TIDE_OK;
}

namespace {
// tide_refresh and tide_refresh_deferred.  Deferred: the selection runs on a copy of the tables, the
// newcomers are copied into staging blobs, and the layer keeps serving from the old placement until
// tide_commit moves the staged blobs into their slots and swaps the tables.
int refresh_impl(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts,
                 int32_t* resident_out, tide_copy* plan_out, int* n_copies_out, void* hip_stream, bool deferred,
                 bool async = false) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (capacity < 0 || capacity > ctx->cfg.capacity) return fail(ctx, TIDE_E_RANGE, "capacity %d outside 0..%d", capacity, ctx->cfg.capacity);
    Layer& L = ctx->layers[layer];
    if (!L.host_blobs) return fail(ctx, TIDE_E_STATE, "layer %d: experts not registered", layer);
    if (!L.placed) return fail(ctx, TIDE_E_STATE, "layer %d has no placement: call tide_set_resident first", layer);
    if (ctx->shape.resident_p12 && !L.comp_blobs)
        return fail(ctx, TIDE_E_STATE, "layer %d: 12-bit slots need the compressed blobs (tide_register_compressed)", layer);
    if (L.deferred_pending) return fail(ctx, TIDE_E_STATE, "layer %d: a deferred refresh awaits tide_commit", layer);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint64_t bytes = tide_expert_blob_bytes(&ctx->cfg);
    if (deferred && !L.staging) {
        void* p = nullptr;
        if (hipMalloc(&p, bytes * (uint64_t)ctx->cfg.capacity) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, TIDE_E_NOMEM, "out of device memory for %d staging blobs", ctx->cfg.capacity);
        }
        L.staging = static_cast<uint8_t*>(p);
        if (hipMalloc(&p, (size_t)(ctx->cfg.n_experts + ctx->cfg.capacity) * sizeof(int32_t)) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, TIDE_E_NOMEM, "out of device memory for the pending tables");
        }
        L.pend_slot_of = static_cast<int32_t*>(p);
        L.pend_eis = L.pend_slot_of + ctx->cfg.n_experts;
    }
    const int32_t* counts = L.t.hits;
    if (counts_host) {
        TIDE_HIP(ctx, hipMemcpyAsync(ctx->ws.counts_tmp, counts_host, ctx->cfg.n_experts * 4, hipMemcpyHostToDevice, stream));
        counts = ctx->ws.counts_tmp;
    }
    // copies of an earlier refresh must have landed before their slots can be given away again
    if (L.copies_recorded) TIDE_HIP(ctx, hipStreamWaitEvent(stream, L.copies_done, 0));
    LayerTables sel = L.t;
    if (deferred) {
        TIDE_HIP(ctx, hipMemcpyAsync(L.pend_slot_of, L.t.slot_of, (size_t)ctx->cfg.n_experts * 4, hipMemcpyDeviceToDevice, stream));
        TIDE_HIP(ctx, hipMemcpyAsync(L.pend_eis, L.t.expert_in_slot, (size_t)ctx->cfg.capacity * 4, hipMemcpyDeviceToDevice, stream));
        sel.slot_of = L.pend_slot_of;
        sel.expert_in_slot = L.pend_eis;
    }
    TIDE_HIP(ctx, launch_refresh_select(ctx->shape, sel, counts, capacity, reset_counts, L.plan, stream));
    uint8_t* copy_dst = deferred ? L.staging : reinterpret_cast<uint8_t*>(L.slots_owned);
    int n = -1;
    if (async) {
        // nothing here needs the plan on the host: the copy kernels read it, and the number of copies, from the pinned
        // block the selection wrote.  The side stream waits for the selection, hence for every earlier step that could
        // still read a slot about to be overwritten.
        TIDE_HIP(ctx, hipEventRecord(L.select_done, stream));
        TIDE_HIP(ctx, hipStreamWaitEvent(ctx->side, L.select_done, 0));
    } else {
        // the plan goes back to the caller; this also means every earlier step that could still read a slot (or a
        // staging blob) about to be overwritten has finished
        TIDE_HIP(ctx, hipStreamSynchronize(stream));
        n = L.plan->n_copies;
    }
    L.result_pending = async;
    TIDE_HIP(ctx, hipEventRecord(L.copies_begin, ctx->side));
    if (ctx->copy_engine == TIDE_COPY_DMA && !async) {
        // one DMA transfer per entering expert, raw blob to slot (or staging blob): the copy engines move the bytes,
        // no compute unit is involved, so kernels that run beside the copies keep their memory pipelines to themselves
        for (int i = 0; i < n; ++i) {
            const BlobSource src = resident_source(ctx, L, L.plan->expert[i]);
            TIDE_HIP(ctx, hipMemcpyAsync(copy_dst + (uint64_t)(deferred ? i : L.plan->slot[i]) * bytes, src.ptr, src.bytes,
                                         hipMemcpyHostToDevice, ctx->side));
        }
    } else if (L.comp_blobs)
        TIDE_HIP(ctx, launch_refresh_copies_p12(L.comp_blobs, L.comp_stride, L.host_blobs, L.host_stride, bytes, copy_dst, L.plan, n,
                                                deferred, ctx->shape.resident_p12 != 0, ctx->shape.d, ctx->shape.I, ctx->side));
    else
        TIDE_HIP(ctx, launch_refresh_copies(L.host_blobs, L.host_stride, bytes, copy_dst, L.plan, n, deferred, ctx->side));
    if (async) {
        TIDE_HIP(ctx, hipEventRecord(L.copies_done, ctx->side));
        L.copies_recorded = true;
        L.copies_pending = true;
        return TIDE_OK;
    }
    for (int i = 0; i < n; ++i) {
        const int e = L.plan->expert[i], s = L.plan->slot[i];
        if (plan_out) {
            plan_out[i].expert = e;
            plan_out[i].slot = s;
            plan_out[i].host_offset = (uint64_t)e * L.host_stride;
            plan_out[i].bytes = bytes;
        }
        if (deferred) L.pend_slots.push_back(s);
    }
    TIDE_HIP(ctx, hipEventRecord(L.copies_done, ctx->side));
    L.copies_recorded = true;
    if (deferred) L.deferred_pending = true;
    else L.copies_pending = n > 0;
    if (n_copies_out) *n_copies_out = n;
    if (resident_out) memcpy(resident_out, L.plan->expert_in_slot, ctx->cfg.capacity * sizeof(int32_t));
    return TIDE_OK;
}
}  // namespace

int tide_refresh(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts,
                 int32_t* resident_out, tide_copy* plan_out, int* n_copies_out, void* hip_stream) {
    return refresh_impl(ctx, layer, counts_host, capacity, reset_counts, resident_out, plan_out, n_copies_out, hip_stream, false);
}

int tide_refresh_async(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts, void* hip_stream) {
    return refresh_impl(ctx, layer, counts_host, capacity, reset_counts, nullptr, nullptr, nullptr, hip_stream, false, true);
}

int tide_refresh_result(tide_ctx* ctx, int layer, int32_t* resident_out, tide_copy* plan_out, int* n_copies_out) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    Layer& L = ctx->layers[layer];
    if (!L.copies_recorded) return fail(ctx, TIDE_E_STATE, "no refresh has run on layer %d", layer);
    if (L.result_pending) TIDE_HIP(ctx, hipEventSynchronize(L.select_done));
    L.result_pending = false;
    const int n = L.plan->n_copies;
    const uint64_t bytes = tide_expert_blob_bytes(&ctx->cfg);
    for (int i = 0; i < n && plan_out; ++i) {
        plan_out[i].expert = L.plan->expert[i];
        plan_out[i].slot = L.plan->slot[i];
        plan_out[i].host_offset = (uint64_t)L.plan->expert[i] * L.host_stride;
        plan_out[i].bytes = bytes;
    }
    if (n_copies_out) *n_copies_out = n;
    if (resident_out) memcpy(resident_out, L.plan->expert_in_slot, ctx->cfg.capacity * sizeof(int32_t));
    return TIDE_OK;
}

int tide_refresh_deferred(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts,
                          int32_t* resident_out, tide_copy* plan_out, int* n_copies_out, void* hip_stream) {
    return refresh_impl(ctx, layer, counts_host, capacity, reset_counts, resident_out, plan_out, n_copies_out, hip_stream, true);
}

int tide_commit(tide_ctx* ctx, int layer, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    Layer& L = ctx->layers[layer];
    if (!L.deferred_pending) return fail(ctx, TIDE_E_STATE, "layer %d: no deferred refresh to commit", layer);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint64_t bytes = tide_expert_blob_bytes(&ctx->cfg);
    // after the host-link copies, and (stream order) after every step that still reads the old slots
    TIDE_HIP(ctx, hipStreamWaitEvent(stream, L.copies_done, 0));
    for (size_t i = 0; i < L.pend_slots.size(); ++i)
        TIDE_HIP(ctx, hipMemcpyAsync(slot_ptr(ctx, L, L.pend_slots[i]), L.staging + (uint64_t)i * bytes, bytes, hipMemcpyDeviceToDevice, stream));
    TIDE_HIP(ctx, hipMemcpyAsync(L.t.slot_of, L.pend_slot_of, (size_t)ctx->cfg.n_experts * 4, hipMemcpyDeviceToDevice, stream));
    TIDE_HIP(ctx, hipMemcpyAsync(L.t.expert_in_slot, L.pend_eis, (size_t)ctx->cfg.capacity * 4, hipMemcpyDeviceToDevice, stream));
    L.pend_slots.clear();
    L.deferred_pending = false;
    return TIDE_OK;
}

int tide_refresh_engine(tide_ctx* ctx, int engine) {
    if (!ctx) return TIDE_E_INVAL;
    if (engine != TIDE_COPY_KERNEL && engine != TIDE_COPY_DMA) return fail(ctx, TIDE_E_INVAL, "engine must be TIDE_COPY_KERNEL or TIDE_COPY_DMA");
    ctx->copy_engine = engine;
    return TIDE_OK;
}

int tide_queue_refresh_wait(tide_ctx* ctx, int layer, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    Layer& L = ctx->layers[layer];
    if (L.copies_recorded) TIDE_HIP(ctx, hipStreamWaitEvent(static_cast<hipStream_t>(hip_stream), L.copies_done, 0));
    return TIDE_OK;
}

int tide_wait_refresh(tide_ctx* ctx, int layer) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    Layer& L = ctx->layers[layer];
    if (L.copies_recorded) TIDE_HIP(ctx, hipEventSynchronize(L.copies_done));
    return TIDE_OK;
}

int tide_refresh_copy_ms(tide_ctx* ctx, int layer, float* ms_out) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!ms_out) return fail(ctx, TIDE_E_INVAL, "ms_out is null");
    Layer& L = ctx->layers[layer];
    if (!L.copies_recorded) return fail(ctx, TIDE_E_STATE, "no refresh has run on layer %d", layer);
    TIDE_HIP(ctx, hipEventSynchronize(L.copies_done));
    TIDE_HIP(ctx, hipEventElapsedTime(ms_out, L.copies_begin, L.copies_done));
    return TIDE_OK;
}

int tide_get_table(tide_ctx* ctx, int layer, int32_t* slot_of_host, void* hip_stream) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!slot_of_host) return fail(ctx, TIDE_E_INVAL, "slot_of_host is null");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TIDE_HIP(ctx, hipMemcpyAsync(slot_of_host, ctx->layers[layer].t.slot_of, ctx->cfg.n_experts * 4, hipMemcpyDeviceToHost, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    return TIDE_OK;
}

int tide_read_slot(tide_ctx* ctx, int layer, int slot, void* blob_host) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (slot < 0 || slot > ctx->cfg.capacity) return fail(ctx, TIDE_E_RANGE, "slot %d outside 0..capacity", slot);
    if (!blob_host) return fail(ctx, TIDE_E_INVAL, "blob_host is null");
    Layer& L = ctx->layers[layer];
    TIDE_HIP(ctx, hipDeviceSynchronize());
    TIDE_HIP(ctx, hipMemcpy(blob_host, slot_ptr(ctx, L, slot), tide_expert_blob_bytes(&ctx->cfg), hipMemcpyDeviceToHost));
    return TIDE_OK;
}

int tide_profile(tide_ctx* ctx, int enable) {
    if (!ctx) return TIDE_E_INVAL;
    TIDE_HIP(ctx, hipDeviceSynchronize());
    ctx->profiling = (enable == 2 || enable == 3) ? enable : (enable != 0 ? 1 : 0);
    ctx->prof_spans.clear();
    ctx->prof_used = 0;
    // events for 512 steps are made here, not inside the region being measured (more are made on demand)
    if (ctx->profiling) {
        const size_t want = (size_t)512 * 2 * TIDE_K_COUNT;
        ctx->prof_spans.reserve(want / 2);
        while (ctx->prof_pool.size() < want) {
            hipEvent_t e = nullptr;
            TIDE_HIP(ctx, hipEventCreate(&e));
            ctx->prof_pool.push_back(e);
        }
    }
    return TIDE_OK;
}

int tide_profile_read(tide_ctx* ctx, double* ms_sum, int64_t* launches) {
    if (!ctx || !ms_sum || !launches) return ctx ? fail(ctx, TIDE_E_INVAL, "null output") : TIDE_E_INVAL;
    TIDE_HIP(ctx, hipDeviceSynchronize());
    for (int i = 0; i < TIDE_K_COUNT; ++i) { ms_sum[i] = 0.0; launches[i] = 0; }
    for (auto& sp : ctx->prof_spans) {
        float ms = 0.f;
        TIDE_HIP(ctx, hipEventElapsedTime(&ms, sp.second.first, sp.second.second));
        ms_sum[sp.first] += ms;
        launches[sp.first] += 1;
    }
    ctx->prof_spans.clear();
    ctx->prof_used = 0;
    return TIDE_OK;
}

int tide_hbm_stream_probe(tide_ctx* ctx, int layer, int repeats, double* gbytes_per_s_host, uint64_t* bytes_host) {
    int rc = layer_ok(ctx, layer);
    if (rc) return rc;
    if (!gbytes_per_s_host || repeats < 1 || repeats > 1000) return fail(ctx, TIDE_E_INVAL, "null output or repeats outside 1..1000");
    Layer& L = ctx->layers[layer];
    const uint64_t bytes = (uint64_t)(ctx->cfg.capacity + ctx->cfg.n_shared) * tide_expert_blob_bytes(&ctx->cfg) / 1024 * 1024;
    hipDeviceProp_t prop;
    TIDE_HIP(ctx, hipGetDeviceProperties(&prop, ctx->device));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    TIDE_HIP(ctx, hipEventCreate(&e0));
    TIDE_HIP(ctx, hipEventCreate(&e1));
    TIDE_HIP(ctx, hipDeviceSynchronize());
    double best_ms = 0.0, sum_ms = 0.0;
    for (int r = 0; r < repeats + 1; ++r) {                     // the first launch is a warm-up
        LaunchEvents ev;
        ev.start = e0;
        ev.stop = e1;
        hipError_t le = launch_stream_probe(reinterpret_cast<const uint8_t*>(L.slots_owned), bytes, 2 * prop.multiProcessorCount,
                                            reinterpret_cast<uint32_t*>(ctx->ws.counts_tmp), nullptr, ev);
        if (le != hipSuccess) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return fail(ctx, TIDE_E_HIP, "stream probe: %s", hipGetErrorString(le)); }
        TIDE_HIP(ctx, hipDeviceSynchronize());
        float ms = 0.f;
        TIDE_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
        if (r > 0) { sum_ms += ms; best_ms = (best_ms == 0.0 || ms < best_ms) ? ms : best_ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *gbytes_per_s_host = (double)bytes / (sum_ms / repeats * 1e-3) / 1e9;
    if (bytes_host) *bytes_host = bytes;
    return TIDE_OK;
}

int tide_counters(tide_ctx* ctx, int64_t* out4, int reset, void* hip_stream) {
    if (!ctx || !out4) return ctx ? fail(ctx, TIDE_E_INVAL, "null output") : TIDE_E_INVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TIDE_HIP(ctx, hipMemcpyAsync(out4, ctx->ws.counters, 4 * sizeof(int64_t), hipMemcpyDeviceToHost, stream));
    if (reset) TIDE_HIP(ctx, launch_clear_i32(reinterpret_cast<int32_t*>(ctx->ws.counters), 8, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    return TIDE_OK;
}

int tide_scale_counts(tide_ctx* ctx, int layer, int num, int den, void* hip_stream) {
    if (!ctx) return TIDE_E_INVAL;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, TIDE_E_RANGE, "layer %d out of range", layer);
    if (den < 1 || num < 0 || num > den) return fail(ctx, TIDE_E_RANGE, "need 0 <= num <= den, den >= 1");
    TIDE_HIP(ctx, launch_scale_counts(ctx->layers[layer].t.hits, ctx->cfg.n_experts, num, den, static_cast<hipStream_t>(hip_stream)));
    return TIDE_OK;
}

int tide_step_histogram(tide_ctx* ctx, int32_t* counts_host, int n_experts, void* hip_stream) {
    if (!ctx || !counts_host) return ctx ? fail(ctx, TIDE_E_INVAL, "null output") : TIDE_E_INVAL;
    if (n_experts != ctx->cfg.n_experts) return fail(ctx, TIDE_E_RANGE, "n_experts %d != configured %d", n_experts, ctx->cfg.n_experts);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TIDE_HIP(ctx, hipMemcpyAsync(counts_host, ctx->last.hist_step, (size_t)n_experts * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    TIDE_HIP(ctx, hipStreamSynchronize(stream));
    return TIDE_OK;
}

int tide_routing_stability(tide_ctx* ctx, const int32_t* counts_dev, int n_steps, int n_experts, int budget,
                           double* sim_dev, int32_t* unique_dev, double* drift_dev, void* hip_stream) {
    if (!counts_dev) return fail(ctx, TIDE_E_INVAL, "counts_dev is null");
    if (n_steps < 1 || n_steps > 65535) return fail(ctx, TIDE_E_RANGE, "n_steps must be 1..65535");
    if (n_experts < 1 || n_experts > kMaxExperts) return fail(ctx, TIDE_E_RANGE, "n_experts must be 1..%d", kMaxExperts);
    if (drift_dev && (budget < 1 || budget > n_experts)) return fail(ctx, TIDE_E_RANGE, "budget must be 1..n_experts");
    hipError_t e = launch_routing_stability(counts_dev, n_steps, n_experts, budget, sim_dev, unique_dev, drift_dev,
                                            static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(ctx, TIDE_E_HIP, "routing stability kernels: %s", hipGetErrorString(e));
    return TIDE_OK;
}

int tide_interval_costs(int budget, int n_steps, double d, double c_io, double c_cpu, const double* f_host,
                        double* lat_io_host, double* lat_cpu_host) {
    if (!f_host || !lat_io_host || !lat_cpu_host) return fail(nullptr, TIDE_E_INVAL, "null array");
    if (budget < 1 || n_steps < 2) return fail(nullptr, TIDE_E_RANGE, "budget must be >= 1 and n_steps >= 2");
    if (!(d >= 0.0 && d <= 1.0)) return fail(nullptr, TIDE_E_RANGE, "drift rate must be in [0, 1]");
    interval_costs(budget, n_steps, d, c_io, c_cpu, f_host, lat_io_host, lat_cpu_host);
    return TIDE_OK;
}

int tide_optimal_interval(int budget, int n_steps, double d, double c_io, double c_cpu, const double* f_host,
                          int* tau_host, double* cost_host) {
    if (!f_host || !tau_host || !cost_host) return fail(nullptr, TIDE_E_INVAL, "null argument");
    if (budget < 1 || n_steps < 2) return fail(nullptr, TIDE_E_RANGE, "budget must be >= 1 and n_steps >= 2");
    if (!(d >= 0.0 && d <= 1.0)) return fail(nullptr, TIDE_E_RANGE, "drift rate must be in [0, 1]");
    std::vector<double> io(n_steps - 1), cpu(n_steps - 1);
    interval_costs(budget, n_steps, d, c_io, c_cpu, f_host, io.data(), cpu.data());
    int best = 0;
    for (int i = 1; i < n_steps - 1; ++i)
        if (io[i] + cpu[i] < io[best] + cpu[best]) best = i;
    *tau_host = best + 1;
    *cost_host = io[best] + cpu[best];
    return TIDE_OK;
}

int tide_fit_drift(double migrations, int budget, int n_steps, int tau, double* d_host) {
    if (!d_host) return fail(nullptr, TIDE_E_INVAL, "null output");
    if (budget < 1 || n_steps < 1 || tau < 1) return fail(nullptr, TIDE_E_RANGE, "budget, n_steps and tau must be >= 1");
    double frac = migrations * (double)tau / (double)((int64_t)budget * n_steps);
    frac = std::min(std::max(frac, 0.0), 1.0);
    *d_host = 1.0 - std::pow(1.0 - frac, 1.0 / (double)tau);
    return TIDE_OK;
}

}  // extern "C"
