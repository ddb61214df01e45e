// Internal declarations shared by the kernel translation units of libtide.
// Every launcher enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "tide.h"

namespace tide {

constexpr int kMaxExperts = 512;        // E limit: 8 router scores per lane of a 64-wide wave
constexpr int kMaxTokens = 65535;       // tokens per step: the per-token kernels put the token on a 16-bit grid axis
constexpr int kMaxTopK = 16;             // one selection per lane of a 16-lane group
constexpr int kMaxRouterSplits = 8;      // slices of the hidden dimension the router logits are computed in
constexpr int kRowsPerTask = 32;        // rows of a small work item
constexpr int kRowsPerBigTask = 256;    // rows of a large work item (the kernels' limit)
constexpr int kRowsPerBigTaskP12 = 192; // the same when the slots hold the 12-bit form: the decode needs the registers of four token tiles
constexpr int kSharedP12MaxTokens = 64; // 12-bit slots: the shared expert keeps the 12-bit form only in contexts of at most this many tokens per step (its work items then have at most four token tiles; wider ones run faster from bf16)
constexpr int kMinBigUnits = 128;       // a step uses large work items only if they make at least this many gate/up workgroups (half the compute units)
constexpr int kBigMinRows = 32;         // a slot with more rows than this is cut into large work items, else into small ones
// Steps with fewer rows per slot on average launch no large-item kernels at all.  A large unit streams 256 weight rows
// of length d: the shorter they are, the more of the unit is its fixed start and end, and the more rows it takes for
// large items to pay (measured: from about 48 rows per slot at d = 4096, about 150 at d = 2048).
constexpr int kBigMinAvgRows = 48, kBigMinAvgRowsShort = 144, kLongRow = 4096;

// running totals (tide_counters): integer adds, so their order does not matter
__device__ inline void bump(int64_t* counter, int64_t by) {
    atomicAdd(reinterpret_cast<unsigned long long*>(counter), (unsigned long long)by);
}

// One grouped-GEMM work item: rows [row0, row0+nrows) of the slot-sorted row space
// all belong to cache slot `slot` (slot == capacity means the shared expert).
struct Task {
    int32_t slot;
    int32_t row0;
    int32_t nrows;
    int32_t flags;      // kTaskSiblings | kTaskP12
};
constexpr int kTaskSiblings = 1;   // small items: the slot is cut into several items (they read the same weights)
constexpr int kTaskP12 = 2;        // the slot holds the 12-bit form of its blob (packed12.h), not the bf16 blob

// Device-side workspace of one context (shared by its layers; one step at a time).
struct Workspace {
    float*   logits;      // [kMaxRouterSplits][max_tokens][E padded to 16] partial router logits
    int32_t* topk_idx;    // [max_tokens][k]
    float*   topk_w;      // [max_tokens][k]
    int32_t* hist_step;   // [E] hits of the step in flight
    int32_t* row_token;   // [max_rows] token of each slot-sorted row
    int32_t* pair_row;    // [max_tokens*k] row of each (token, rank) pair, -1 = miss
    int32_t* slot_off;    // [capacity+2] first row of each slot (shared slot last), then total rows
    Task*    tasks;       // [max_small_tasks] small work items
    Task*    big_tasks;   // [max_big_tasks] large work items
    int32_t* n_tasks;     // [2] number of small, large work items
    int32_t* big_order;   // [max_big_tasks] large work items, heaviest first
    uint16_t* act;        // [max_rows][d_ff] bf16 SwiGLU activations
    float*   y;           // [max_rows][d] per-row expert outputs
    int32_t* counts_tmp;  // [E] caller-provided counts for a refresh
    int64_t* counters;    // [4] running totals: steps, active slots (shared included), rows, misses
    int32_t* m_idx;       // [max_tokens*k] miss pass: expert, token and weight of each listed miss
    int32_t* m_tok;
    float*   m_w;
    int32_t* miss_hist;   // [E] listed misses per expert
    int32_t* m_count;     // [1] number of listed misses
};

struct LayerTables {
    int32_t* hits;            // H[E]
    int32_t* slot_of;         // [E]  slot of each expert, -1 = not resident
    int32_t* expert_in_slot;  // [capacity] expert in each slot, -1 = empty
    const uint16_t* slots;    // capacity (+1 shared) packed blobs, blob_elems apart
    const uint8_t* expert_p12; // [E + n_shared] 1 = the expert's blob is kept in a slot in its 12-bit form; null: bf16 slots
};

// Optional timing of one kernel launch: when both events are set the launch goes through
// hipExtLaunchKernelGGL, which stamps them with the dispatch's own begin and end times
// (no extra barrier packets in the stream, the kernel's neighbours are not disturbed).
struct LaunchEvents {
    hipEvent_t start = nullptr;
    hipEvent_t stop = nullptr;
};
#define TIDE_LAUNCH(kernel, grid, block, stream, ev, ...)                                                   \
    do {                                                                                                    \
        if ((ev).start && (ev).stop)                                                                        \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, (ev).start, (ev).stop, 0, __VA_ARGS__);   \
        else                                                                                                \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                                \
    } while (0)

struct Shape {
    int d, E, k, I, n_shared, capacity, gating, bias_mode;
    int64_t blob_elems;       // 3*d*I
    int n_cus;                // compute units of the device
    int big_rows;             // most rows of a large work item: kRowsPerBigTask or kRowsPerBigTaskP12
    int resident_p12;         // the cache slots hold the 12-bit form of the blobs (packed12.h)
};
inline int big_min_avg_rows(const Shape& s) { return s.d >= kLongRow ? kBigMinAvgRows : kBigMinAvgRowsShort; }

// a1: z[n][e] = <x_n, W_r[e]>  (fp32)
hipError_t launch_router_logits(const Shape& s, const uint16_t* x, int n_tokens, const float* w_r,
                                float* logits, int32_t* hist_step_to_clear, hipStream_t stream, LaunchEvents ev = {});
// a2 + a3: gate, top-k, weights; hist_step[e] += 1 per selected pair (H += hist_step is launch_dispatch's)
hipError_t launch_topk_gate(const Shape& s, const float* logits, const float* bias, int n_tokens,
                            int32_t* topk_idx, float* topk_w, int32_t* hist_step,
                            int32_t* idx_copy, float* w_copy, hipStream_t stream, LaunchEvents ev = {});
// a2..a5 for a step of at most 32 tokens, in one workgroup: top-k, weights, counts, hit/miss split
bool routes_in_one_workgroup(const Shape& s, int n_tokens);
hipError_t launch_route_small(const Shape& s, const LayerTables& t, const Workspace& w, const float* bias, int n_tokens,
                              int32_t* idx_copy, float* w_copy, tide_miss* miss, int miss_cap, int32_t* n_miss,
                              hipStream_t stream, LaunchEvents ev = {});
// a3 for token states that arrive routed: clear + count into hist_step (H += hist_step is launch_dispatch's)
hipError_t launch_count_pairs(const Shape& s, const int32_t* topk_idx, int n_tokens, int32_t* hist_step,
                              hipStream_t stream);
// p[0..n) = 0 by a fill kernel (safe inside a captured graph, unlike a memset node)
hipError_t launch_clear_i32(int32_t* p, int n, hipStream_t stream);
// a4 + a5: H += hist_step; hit/miss split, canonical miss list, slot-sorted rows, work items
hipError_t launch_dispatch(const Shape& s, const LayerTables& t, const Workspace& w, const int32_t* topk_idx,
                           const float* topk_w, int n_tokens, tide_miss* miss, int miss_cap, int32_t* n_miss,
                           hipStream_t stream, LaunchEvents ev = {});
// a6 / a7 / a8: grouped SwiGLU expert GEMMs over the work items
// pass 0 = gate/up + SwiGLU -> act; pass 1 = down -> y; small and large work items
hipError_t launch_expert_gemm(int pass, const Shape& s, const LayerTables& t, const Workspace& w, const uint16_t* x,
                              int max_tasks, hipStream_t stream, LaunchEvents ev = {});
hipError_t launch_expert_gemm_big(int pass, const Shape& s, const LayerTables& t, const Workspace& w,
                                  const uint16_t* x, int max_big_tasks, hipStream_t stream, LaunchEvents ev = {});
// ranks the large work items heaviest first (w.big_order); runs after the work items are written and
// before launch_expert_gemm_big
hipError_t launch_plan_big(const Workspace& w, int max_big_tasks, hipStream_t stream);
// upper bound of the number of large work items a step over n_tokens tokens can produce
inline int max_big_tasks_for(const Shape& s, int n_tokens) {
    if (n_tokens <= kBigMinRows) return 0;
    const int rows = n_tokens * s.k + (s.n_shared ? n_tokens : 0);
    const int slots = s.capacity + 1;
    const int busy = rows / (kBigMinRows + 1);           // slots that can exceed the small limit at once
    const int most = rows / s.big_rows + (busy < slots ? busy : slots);
    // too few for the step ever to choose large items (the split kernel's rule), or so few rows per slot that the
    // large-item kernels would mostly be launched for nothing (their idle workgroups each take a compute unit's LDS
    // for a moment: 135 -> 123 us per step at 256 tokens x top-8 over 65 slots): nothing to launch, and the split
    // kernel, told so, cuts every slot into small items
    if ((int64_t)most * ((s.I + 127) / 128) < kMinBigUnits || rows < big_min_avg_rows(s) * slots) return 0;
    return most;
}
// upper bound of the number of small work items
inline int max_small_tasks_for(const Shape& s, int n_tokens) {
    const int rows = n_tokens * s.k + (s.n_shared ? n_tokens : 0);
    return s.capacity + 1 + rows / kRowsPerTask;
}
// the same bounds for a miss pass, whose groups are the E experts instead of the cache slots
inline int max_miss_small_tasks_for(const Shape& s, int n_tokens) { return s.E + n_tokens * s.k / kRowsPerTask; }
inline int max_miss_big_tasks_for(const Shape& s, int n_tokens) {
    if (n_tokens <= kBigMinRows) return 0;
    const int rows = n_tokens * s.k;
    const int busy = rows / (kBigMinRows + 1);
    const int most = rows / s.big_rows + (busy < s.E ? busy : s.E);
    if ((int64_t)most * ((s.I + 127) / 128) < kMinBigUnits || rows < big_min_avg_rows(s) * s.E) return 0;
    return most;
}
// miss pass (the step's misses evaluated from the host-resident blobs; entries that name an expert outside [0,E)
// or a token outside [0,n_tokens) are skipped): group the list by expert into
// rows and work items whose "slot" is the expert id; add the weighted results to out
// expert_mask (device or pinned host, [E] bytes, may be null): only experts with a non-zero byte are evaluated
hipError_t launch_miss_group(const Shape& s, const Workspace& w, const tide_miss* miss, int miss_cap,
                             const int32_t* n_miss, int n_tokens, int max_big, hipStream_t stream,
                             const uint8_t* expert_mask = nullptr);
hipError_t launch_miss_combine(const Shape& s, const Workspace& w, int n_tokens, float* out, hipStream_t stream);
// a9: out[n] = shared row + sum over hit pairs in rank order of w * y[row]
hipError_t launch_combine(const Shape& s, const Workspace& w, const float* topk_w, int n_tokens, float* out,
                          hipStream_t stream, LaunchEvents ev = {});
// the first min(*n_miss, cap) list entries, their number and the token states they name -> pinned host memory
hipError_t launch_miss_export(const tide_miss* miss, int cap, const int32_t* n_miss, const uint16_t* x, int n_tokens,
                              int d, tide_miss* miss_host, int32_t* n_host, uint16_t* x_host, hipStream_t stream);
// out[tokens[r]] += rows[r] for n_rows rows of d floats (rows / tokens: device or pinned host memory)
hipError_t launch_add_rows(const float* rows, const int32_t* tokens, int n_rows, int d, float* out, hipStream_t stream);
// a11: top-capacity selection + slot plan, tables updated in place
struct RefreshOut {           // lives in pinned host memory the kernel writes directly
    int32_t n_copies;
    int32_t pad;
    int32_t expert[kMaxExperts];
    int32_t slot[kMaxExperts];
    int32_t expert_in_slot[kMaxExperts];
};
hipError_t launch_refresh_select(const Shape& s, const LayerTables& t, const int32_t* counts, int capacity,
                                 int reset_counts, RefreshOut* out_hostmapped, hipStream_t stream);

// a12: the plan's blobs from pinned host memory to their slots (or to staging blob i), one kernel.  n < 0: the
// kernel takes the number of copies from the plan itself (the host has not seen it)
hipError_t launch_refresh_copies(const uint8_t* host_blobs, uint64_t host_stride, uint64_t blob_bytes, uint8_t* dst_base,
                                 const RefreshOut* plan, int n, bool dst_by_rank, hipStream_t stream);
// the same copies from the 12-bit form of the blobs (packed12.h): rebuilt bit for bit in the destination, or
// (verbatim) copied as they are for slots that keep the 12-bit form
hipError_t launch_refresh_copies_p12(const uint8_t* comp_blobs, uint64_t comp_stride, const uint8_t* host_blobs,
                                     uint64_t host_stride, uint64_t blob_bytes, uint8_t* dst_base, const RefreshOut* plan, int n,
                                     bool dst_by_rank, bool verbatim, int d, int d_ff, hipStream_t stream);
// measurement: `bytes` (a multiple of 1024) from `base` read once by `workgroups` workgroups in the GEMMs' weight-stream shape
hipError_t launch_stream_probe(const uint8_t* base, uint64_t bytes, int workgroups, uint32_t* sink, hipStream_t stream, LaunchEvents ev);
// H[e] <- floor(H[e] * num / den)
hipError_t launch_scale_counts(int32_t* hits, int n_experts, int num, int den, hipStream_t stream);
// interval analysis (Sec. 3.2, Eq. 4-7): similarity / distinct experts / drift on the device, cost model on the host
hipError_t launch_routing_stability(const int32_t* counts, int n_steps, int n_experts, int budget, double* sim,
                                    int32_t* unique, double* drift, hipStream_t stream);
void interval_costs(int budget, int n_steps, double d, double c_io, double c_cpu, const double* f, double* lat_io,
                    double* lat_cpu);

// Packed blob: the gate and up matrices interleaved (2*d*I elements), then the down matrix (d*I).
// Stripes (16 matrix rows) are stored in groups, K chunk slow inside a group (tide_pack_expert).
constexpr int kGateUpGroup = 8;     // SwiGLU column blocks (a gate and an up stripe each) per group
constexpr int kDownGroup = 16;      // down stripes per group
inline int64_t blob_off_gate_up(const Shape&) { return 0; }
inline int64_t blob_off_down(const Shape& s) { return 2 * (int64_t)s.d * s.I; }

}  // namespace tide
