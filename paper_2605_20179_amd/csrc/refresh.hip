// Refresh step: the resident set becomes the current top-B experts by hit count
// (Alg. 1 refresh step: most-hit CPU experts in, least-hit GPU experts out; Sec. 3.3).
// One workgroup, one expert per thread, all-pairs ranking (E <= 512).
#include "tide_internal.h"

namespace tide {

namespace {

constexpr int kThreads = kMaxExperts;

__global__ __launch_bounds__(kThreads) void refresh_select_kernel(int n_experts, int n_slots, int capacity,
                                                                  const int32_t* __restrict__ counts,
                                                                  int32_t* __restrict__ hits_to_reset,
                                                                  int32_t* __restrict__ slot_of,
                                                                  int32_t* __restrict__ expert_in_slot,
                                                                  RefreshOut* __restrict__ out) {
    __shared__ int h[kMaxExperts];          // hits
    __shared__ int slot[kMaxExperts];       // slot of expert or -1
    __shared__ int cls[kMaxExperts];        // 0 stays out / stays in, 1 leaving, 2 entering
    __shared__ int free_slot[kMaxExperts];  // freed slots in leaving order, then empty slots ascending
    __shared__ int n_leaving_s, n_entering_s;
    const int e = threadIdx.x;
    const bool live = e < n_experts;
    if (live) {
        h[e] = counts[e];
        slot[e] = slot_of[e];
    }
    if (e == 0) { n_leaving_s = 0; n_entering_s = 0; }
    __syncthreads();

    // rank under (hits descending, resident first, lower id first)
    int my_cls = 0;
    if (live) {
        const int he = h[e];
        const int re = slot[e] >= 0 ? 0 : 1;
        int rank = 0;
        for (int o = 0; o < n_experts; ++o) {
            const int ho = h[o];
            const int ro = slot[o] >= 0 ? 0 : 1;
            const bool before = (ho > he) || (ho == he && (ro < re || (ro == re && o < e)));
            rank += before ? 1 : 0;
        }
        const bool in_new = rank < capacity;
        if (re == 0 && !in_new) my_cls = 1;
        if (re == 1 && in_new) my_cls = 2;
        cls[e] = my_cls;
    }
    __syncthreads();

    // order inside the leaving set: (hits ascending, id); inside the entering set: (hits descending, id)
    int my_pos = -1;
    if (live && my_cls != 0) {
        const int he = h[e];
        int pos = 0;
        for (int o = 0; o < n_experts; ++o) {
            if (cls[o] != my_cls) continue;
            const int ho = h[o];
            const bool before = (my_cls == 1) ? ((ho < he) || (ho == he && o < e)) : ((ho > he) || (ho == he && o < e));
            pos += before ? 1 : 0;
        }
        my_pos = pos;
        atomicAdd(my_cls == 1 ? &n_leaving_s : &n_entering_s, 1);
    }
    __syncthreads();
    const int n_leaving = n_leaving_s, n_entering = n_entering_s;

    if (live && my_cls == 1) free_slot[my_pos] = slot[e];
    // thread s < n_slots looks at slot s: originally empty slots follow the freed ones
    if (e < n_slots && expert_in_slot[e] < 0) {
        int before = 0;
        for (int q = 0; q < e; ++q) before += expert_in_slot[q] < 0 ? 1 : 0;
        free_slot[n_leaving + before] = e;
    }
    __syncthreads();

    if (live && my_cls == 1) {
        expert_in_slot[slot[e]] = -1;
        slot_of[e] = -1;
    }
    __syncthreads();
    if (live && my_cls == 2) {
        const int s = free_slot[my_pos];
        expert_in_slot[s] = e;
        slot_of[e] = s;
        out->expert[my_pos] = e;
        out->slot[my_pos] = s;
    }
    if (live && hits_to_reset != nullptr) hits_to_reset[e] = 0;
    __syncthreads();
    if (e < n_slots) out->expert_in_slot[e] = expert_in_slot[e];
    if (e == 0) {
        out->n_copies = n_entering;
        out->pad = 0;
    }
}

}  // namespace

hipError_t launch_refresh_select(const Shape& s, const LayerTables& t, const int32_t* counts, int capacity,
                                 int reset_counts, RefreshOut* out_hostmapped, hipStream_t stream) {
    hipLaunchKernelGGL(refresh_select_kernel, dim3(1), dim3(kThreads), 0, stream, s.E, s.capacity, capacity, counts,
                       reset_counts ? t.hits : (int32_t*)nullptr, t.slot_of, t.expert_in_slot, out_hostmapped);
    return hipGetLastError();
}

}  // namespace tide
