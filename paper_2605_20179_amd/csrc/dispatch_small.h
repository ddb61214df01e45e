// Hit/miss split for a small step (at most 32 tokens and 1024 (token, expert) pairs), run by a
// single workgroup of kRouteThreads threads right after it has routed the step: same lists, same order and
// same counters as dispatch_kernel produces with one block per slot.
#pragma once
#include "tide_internal.h"

namespace tide {

constexpr int kRouteThreads = 512;               // 16 lanes per token x 32 tokens: two waves per SIMD
constexpr int kSmallDispatchMaxPairs = 1024;
constexpr int kSmallDispatchMaxTokens = 32;      // token sets are 32-bit masks
static_assert(kSmallDispatchMaxTokens <= kBigMinRows && kSmallDispatchMaxTokens <= kRowsPerTask,
              "a small step must never produce a large work item or a slot of more than one item");
constexpr int kSmallDispatchLdsInts = 3 * (kMaxExperts + 8);

struct DispatchArgs {
    int n_tokens, k, capacity, n_shared, n_experts;
    const int32_t* slot_of;
    const int32_t* expert_in_slot;
    const uint8_t* expert_p12;     // LayerTables::expert_p12
    int32_t* row_token;
    int32_t* pair_row;
    int32_t* slot_off;
    Task* tasks;
    int32_t* n_tasks;
    tide_miss* miss;
    int miss_cap;
    int32_t* n_miss;
    int64_t* counters;
};

// s_mask[E]: for every expert the set of tokens that selected it (bit n = token n), which gives both
// the step's histogram (popcount) and, because a token selects an expert at most once, the rank of a
// pair among its slot's rows (popcount of the lower bits) without any ordering pass;
// s_slot_of[E], s_eis[capacity]: the placement tables; s_idx / s_w [n_tokens*k]: the routing; all in
// LDS and complete (the caller has synchronised).  lds: kSmallDispatchLdsInts ints of scratch.
__device__ inline void dispatch_small(const DispatchArgs& a, const unsigned* s_mask, const int* s_slot_of,
                                      const int* s_eis, const int* s_idx, const float* s_w, int* lds) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_pairs = a.n_tokens * a.k;
    const int n_slots = a.capacity + 1;                      // the shared expert is the last slot
    int* s_m = lds;                                          // rows per slot
    int* s_row0 = s_m + kMaxExperts + 8;                     // first row of each slot
    int* s_task0 = s_row0 + kMaxExperts + 8;                 // first work item of each slot

    for (int s = tid; s < n_slots; s += kRouteThreads) {
        int m;
        if (s == a.capacity) {
            m = a.n_shared ? a.n_tokens : 0;
        } else {
            const int e = s_eis[s];
            m = e >= 0 ? __popc(s_mask[e]) : 0;
        }
        s_m[s] = m;
    }
    __syncthreads();

    // exclusive prefix sums over the slots by wave 0: each lane owns a contiguous run of slots
    if (wave == 0) {
        const int per = (n_slots + 63) / 64;
        int rows = 0, items = 0, active = 0;
        for (int i = 0; i < per; ++i) {
            const int s = lane * per + i;
            if (s < n_slots) {
                rows += s_m[s];
                items += (s_m[s] + kRowsPerTask - 1) / kRowsPerTask;
                active += s_m[s] > 0 ? 1 : 0;
            }
        }
        int rows_inc = rows, items_inc = items, active_inc = active;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int r = __shfl_up(rows_inc, off), t = __shfl_up(items_inc, off), c = __shfl_up(active_inc, off);
            if (lane >= off) { rows_inc += r; items_inc += t; active_inc += c; }
        }
        int row0 = rows_inc - rows, task0 = items_inc - items;
        for (int i = 0; i < per; ++i) {
            const int s = lane * per + i;
            if (s < n_slots) {
                s_row0[s] = row0;
                s_task0[s] = task0;
                row0 += s_m[s];
                task0 += (s_m[s] + kRowsPerTask - 1) / kRowsPerTask;
            }
        }
        if (lane == 63) {
            a.slot_off[n_slots] = rows_inc;
            a.n_tasks[0] = items_inc;
            a.n_tasks[1] = 0;                                // at most 32 tokens: no slot can exceed a small item
            bump(a.counters + 0, 1);
            bump(a.counters + 1, active_inc);
            bump(a.counters + 2, rows_inc);
        }
    }
    __syncthreads();

    // work items and slot offsets
    for (int s = tid; s < n_slots; s += kRouteThreads) {
        a.slot_off[s] = s_row0[s];
        const int m = s_m[s];
        const int items = (m + kRowsPerTask - 1) / kRowsPerTask;
        const int e = s < a.capacity ? s_eis[s] : a.n_experts;
        const int fmt_flags = (items && a.expert_p12 && e >= 0 && a.expert_p12[e]) ? kTaskP12 : 0;
        for (int c = 0; c < items; ++c) {
            Task t;
            t.slot = s;
            t.row0 = s_row0[s] + c * kRowsPerTask;
            t.nrows = min(kRowsPerTask, m - c * kRowsPerTask);
            t.flags = fmt_flags;
            a.tasks[s_task0[s] + c] = t;
        }
    }
    // shared expert: every token in token order
    if (a.n_shared)
        for (int n = tid; n < a.n_tokens; n += kRouteThreads) a.row_token[s_row0[a.capacity] + n] = n;

    // hit pairs: row = first row of the slot + number of lower-numbered tokens that chose the expert
    for (int p = tid; p < n_pairs; p += kRouteThreads) {
        const int e = s_idx[p];
        const int slot = (e < 0 || e >= a.n_experts) ? -1 : s_slot_of[e];
        if (slot >= 0) {
            const int n = p / a.k;
            const int row = s_row0[slot] + __popc(s_mask[e] & ((1u << n) - 1u));
            a.row_token[row] = n;
            a.pair_row[p] = row;
        }
    }
    // misses in canonical order (token, then rank): one wave walks the pairs
    if (wave == 3) {
        int running = 0;
        for (int base = 0; base < n_pairs; base += 64) {
            const int p = base + lane;
            int e = -1;
            bool flag = false;
            if (p < n_pairs) {
                e = s_idx[p];
                flag = (e < 0 || e >= a.n_experts) ? true : s_slot_of[e] < 0;
            }
            const unsigned long long b = __ballot(flag);
            if (flag) {
                a.pair_row[p] = -1;
                const int pos = running + __popcll(b & ((1ull << lane) - 1ull));
                if (pos < a.miss_cap) {
                    tide_miss m;
                    m.token = p / a.k;
                    m.expert = e;
                    m.weight = s_w[p];
                    a.miss[pos] = m;
                }
            }
            running += __popcll(b);
        }
        if (lane == 0) {
            *a.n_miss = running;
            bump(a.counters + 3, running);
        }
    }
}

}  // namespace tide
