// Hit/miss split of the step's (token, expert) pairs against the resident table,
// canonical miss list, slot-sorted row lists and grouped-GEMM work items
// (Alg. 1 token routing: pairs whose expert is in E^GPU are computed here, pairs whose
// expert is in E^CPU are handed back).  No atomics: every list is produced by an
// ordered block-level compaction, so results are identical from run to run.
#include "tide_internal.h"

namespace tide {

namespace {

constexpr int kThreads = 1024;

__device__ inline int block_sum(int v, int* lds4) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) t += lds4[w];
    __syncthreads();
    return t;
}

// a and b summed over the block (fields packed by the caller must not overflow into each other).
__device__ inline void block_sum2(unsigned long long& a, unsigned long long& b, unsigned long long* lds8) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off);
        b += __shfl_xor(b, off);
    }
    if ((threadIdx.x & 63) == 0) {
        lds8[2 * (threadIdx.x >> 6)] = a;
        lds8[2 * (threadIdx.x >> 6) + 1] = b;
    }
    __syncthreads();
    a = 0;
    b = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        a += lds8[2 * w];
        b += lds8[2 * w + 1];
    }
    __syncthreads();
}

// ids[0..3] = idx[p0 .. p0+3] (16-byte load when the four are in range; idx is 16-byte aligned).
__device__ inline void load4(const int32_t* __restrict__ idx, int p0, int n, int (&ids)[4]) {
    if (p0 + 3 < n) {
        const int4 v = *reinterpret_cast<const int4*>(idx + p0);
        ids[0] = v.x; ids[1] = v.y; ids[2] = v.z; ids[3] = v.w;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) ids[q] = p0 + q < n ? idx[p0 + q] : -1;
    }
}

// Exclusive prefix sum of v over the block in thread order, and the block total.
__device__ inline int block_scan_excl(int v, int& total, int* lds4) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) lds4[wv] = inc;
    __syncthreads();
    int base = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const int c = lds4[w];
        if (w < wv) base += c;
        total += c;
    }
    __syncthreads();
    return base + inc - v;
}

// A group (cache slot, or expert in a miss pass) with more than kBigMinRows rows is cut into large work
// items of up to kRowsPerBigTask rows -- when the step has enough of them: the large kernels run one
// workgroup per compute unit, so with fewer units than compute units most of the chip would idle and the
// small kernels (several workgroups per compute unit, the second reader of a weight tile served by L2)
// are the faster way.  use_big is the same in every block of a launch.
__device__ inline int n_small_items(int m, bool use_big) {
    return (m <= kBigMinRows || !use_big) ? (m + kRowsPerTask - 1) / kRowsPerTask : 0;
}
__device__ inline int n_big_items(int m, bool use_big, int big_rows) {
    return (m > kBigMinRows && use_big) ? (m + big_rows - 1) / big_rows : 0;
}

// Work items of one slot whose m rows start at row0.
__device__ inline void emit_tasks(int slot, int row0, int m, bool use_big, Task* small_out, Task* big_out, int big_room, int fmt_flags,
                                  int big_rows) {
    if (m <= 0) return;
    if (m <= kBigMinRows || !use_big) {
        const int ns = (m + kRowsPerTask - 1) / kRowsPerTask;
        for (int c = threadIdx.x; c < ns; c += kThreads) {
            Task t;
            t.slot = slot;
            t.row0 = row0 + c * kRowsPerTask;
            t.nrows = min(kRowsPerTask, m - c * kRowsPerTask);
            t.flags = (ns > 1 ? kTaskSiblings : 0) | fmt_flags;      // several items stream the slot's weights: let them meet in L2
            small_out[c] = t;
        }
        return;
    }
    // the fewest large work items that hold m rows, of even size (a whole number of 16-token tiles):
    // 300 rows become 160 + 140, not 256 + 44, so the slot's work items finish together
    const int nb = (m + big_rows - 1) / big_rows;
    const int per = ((m + nb - 1) / nb + 15) / 16 * 16;      // <= big_rows (a multiple of 16), and (nb-1)*per < m
    // the host's bound on the step's large work items holds for any routing (rows / 256 plus one per slot that can
    // exceed the small limit), so big_room >= nb; the clamp only keeps a bound that was computed for another token
    // count from ever turning into a write out of bounds
    for (int c = threadIdx.x; c < nb && c < big_room; c += kThreads) {
        Task t;
        t.slot = slot;
        t.row0 = row0 + c * per;
        t.nrows = min(per, m - c * per);
        t.flags = fmt_flags;
        big_out[c] = t;
    }
}

// Rows of one group: the pairs p (in pair order) whose expert id is e get rows row_begin, row_begin+1, ...
// PAIR_TOKEN: the token of pair p is pair_token[p] (a miss list) instead of p / k (a routing table).
template <bool PAIR_TOKEN>
__device__ inline void collect_rows(const int32_t* __restrict__ idx, const int32_t* __restrict__ pair_token, int n_pairs,
                                    int k, int e, int row_begin, int32_t* __restrict__ row_token,
                                    int32_t* __restrict__ pair_row, int* lds4) {
    const int tid = threadIdx.x;
    int running = 0;
    int next[4];
    load4(idx, 4 * tid, n_pairs, next);                      // the next pass's ids are always in flight
    for (int base = 0; base < n_pairs; base += 4 * kThreads) {
        const int p0 = base + 4 * tid;
        int ids[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) ids[q] = next[q];
        load4(idx, p0 + 4 * kThreads, n_pairs, next);
        bool flag[4];
        int c = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            flag[q] = p0 + q < n_pairs && ids[q] == e;
            c += flag[q] ? 1 : 0;
        }
        int total;
        int row = row_begin + running + block_scan_excl(c, total, lds4);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (flag[q]) {
                row_token[row] = PAIR_TOKEN ? pair_token[p0 + q] : (p0 + q) / k;
                pair_row[p0 + q] = row;
                ++row;
            }
        }
        running += total;
    }
}

// grid = capacity + 2 blocks: one per cache slot, one for the shared expert, one for the misses.
__global__ __launch_bounds__(kThreads) void dispatch_kernel(
    const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w, int n_tokens, int k, int capacity,
    int n_shared, int n_experts, const int32_t* __restrict__ slot_of, const int32_t* __restrict__ expert_in_slot,
    const uint8_t* __restrict__ expert_p12, const int32_t* __restrict__ hist_step, int32_t* __restrict__ hits, int32_t* __restrict__ row_token,
    int32_t* __restrict__ pair_row, int32_t* __restrict__ slot_off, Task* __restrict__ tasks, Task* __restrict__ big_tasks,
    int32_t* __restrict__ n_tasks,
    tide_miss* __restrict__ miss, int miss_cap, int32_t* __restrict__ n_miss, int64_t* __restrict__ counters,
    int max_big, int big_ftiles, int big_rows) {
    __shared__ int lds4[kThreads / 64];
    __shared__ unsigned long long lds8[2 * (kThreads / 64)];
    __shared__ int own[2];                   // this block's slot: expert and rows
    const int s = blockIdx.x;
    const int tid = threadIdx.x;
    const int n_pairs = n_tokens * k;

    if (s == capacity + 1) {
        // misses, ordered by token then rank; each thread takes 4 consecutive pairs per pass
        int running = 0;
        for (int base = 0; base < n_pairs; base += 4 * kThreads) {
            const int p0 = base + 4 * tid;
            int e[4];
            bool flag[4];
            load4(topk_idx, p0, n_pairs, e);
            int c = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // an id outside [0,E) can only come from caller-supplied routing: report it as a miss
                flag[q] = p0 + q < n_pairs && ((e[q] < 0 || e[q] >= n_experts) ? true : slot_of[e[q]] < 0);
                c += flag[q] ? 1 : 0;
            }
            int total;
            int pos = running + block_scan_excl(c, total, lds4);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (flag[q]) {
                    const int p = p0 + q;
                    pair_row[p] = -1;
                    if (pos < miss_cap) {
                        tide_miss m;
                        m.token = p / k;
                        m.expert = e[q];
                        m.weight = topk_w[p];
                        miss[pos] = m;
                    }
                    ++pos;
                }
            }
            running += total;
        }
        if (tid == 0) {
            *n_miss = running;
            bump(counters + 3, running);
        }
        return;
    }

    // One thread per slot (capacity <= kMaxExperts <= kThreads) reads the slot's row count; a single block-wide
    // sum of packed fields then gives everything that precedes this block's slot -- rows, work items, active
    // slots -- and the large work items of the whole step (the same figure in every block).  The small-item
    // count is carried for both outcomes of the step's small/large rule, which depends on that figure.
    static_assert(kMaxExperts <= kThreads, "one thread per cache slot");
    const int upto = s < capacity ? s : capacity;
    unsigned long long fa = 0, fb = 0;
    if (tid < capacity) {
        const int e = expert_in_slot[tid];
        const int m = e >= 0 ? hist_step[e] : 0;
        const unsigned long long big = n_big_items(m, true, big_rows);
        if (tid == s) {
            own[0] = e;
            own[1] = m;
        }
        fa = big;                                                        // bits 0-15: large items, all slots
        if (tid < upto) {
            fa |= (unsigned long long)(m > 0 ? 1 : 0) << 16 | (unsigned long long)m << 32;
            fb = (unsigned long long)n_small_items(m, true) | (unsigned long long)n_small_items(m, false) << 21 | big << 42;
        }
    }
    block_sum2(fa, fb, lds8);
    const int all_big = (int)(fa & 0xffff) + n_big_items(n_shared ? n_tokens : 0, true, big_rows);
    const bool use_big = max_big > 0 && all_big * big_ftiles >= kMinBigUnits;      // max_big == 0: the host launches no large-item kernels
    const int active_before = (int)(fa >> 16 & 0xffff);
    const int rows_before = (int)(fa >> 32);
    const int tasks_before = use_big ? (int)(fb & 0x1fffff) : (int)(fb >> 21 & 0x1fffff);
    const int big_before = use_big ? (int)(fb >> 42) : 0;

    if (s == capacity) {
        // the interval counter takes the step's histogram (Fig. 1 caption: every selected expert counts,
        // resident or not); this block is the step's only writer of H
        for (int e = tid; e < n_experts; e += kThreads) hits[e] += hist_step[e];
        // shared expert: every token, in token order
        const int m = n_shared ? n_tokens : 0;
        for (int n = tid; n < m; n += kThreads) row_token[rows_before + n] = n;
        const int n_small = n_small_items(m, use_big);
        const int n_big = n_big_items(m, use_big, big_rows);
        emit_tasks(capacity, rows_before, m, use_big, tasks + tasks_before, big_tasks + big_before, max_big - big_before,
                   expert_p12 && expert_p12[n_experts] ? kTaskP12 : 0, big_rows);
        if (tid == 0) {
            slot_off[capacity] = rows_before;
            slot_off[capacity + 1] = rows_before + m;
            n_tasks[0] = tasks_before + n_small;
            n_tasks[1] = min(big_before + n_big, max_big);
        }
        if (tid == 0) {
            // running totals for throughput accounting (atomic: the layers of a stack step run on several streams)
            bump(counters + 0, 1);
            bump(counters + 1, active_before + (m > 0 ? 1 : 0));
            bump(counters + 2, rows_before + m);
        }
        return;
    }

    const int e = own[0], m = own[1];        // written before block_sum2's barriers
    if (tid == 0) slot_off[s] = rows_before;
    if (m == 0) return;
    emit_tasks(s, rows_before, m, use_big, tasks + tasks_before, big_tasks + big_before, max_big - big_before,
               expert_p12 && expert_p12[e] ? kTaskP12 : 0, big_rows);
    collect_rows<false>(topk_idx, nullptr, n_pairs, k, e, rows_before, row_token, pair_row, lds4);
}

// ---- miss pass: the miss list of a step, evaluated from the host-resident expert blobs -------------

// Struct-of-arrays copy of the (possibly truncated) miss list and the number of misses per expert.
// With a mask only the entries of experts e with mask[e] != 0 are kept.
__global__ __launch_bounds__(kThreads) void miss_prepare_kernel(const tide_miss* __restrict__ miss, int miss_cap,
                                                               const int32_t* __restrict__ n_miss, int n_experts,
                                                               int n_tokens, const uint8_t* __restrict__ mask,
                                                               int32_t* __restrict__ m_idx, int32_t* __restrict__ m_tok,
                                                               float* __restrict__ m_w, int32_t* __restrict__ miss_hist,
                                                               int32_t* __restrict__ m_count) {
    const int n = min(*n_miss, miss_cap);
    const int p = blockIdx.x * kThreads + threadIdx.x;
    if (p == 0) *m_count = n;
    if (p >= n) return;
    const tide_miss m = miss[p];
    const bool ok = m.expert >= 0 && m.expert < n_experts && m.token >= 0 && m.token < n_tokens &&
                    (mask == nullptr || mask[m.expert] != 0);
    m_idx[p] = ok ? m.expert : -1;                           // an entry out of range or masked out is skipped
    m_tok[p] = m.token;
    m_w[p] = m.weight;
    if (ok) atomicAdd(&miss_hist[m.expert], 1);
}

// grid = E + 1 blocks: block e lists the rows of expert e (the "slot" of a miss-pass work item is the
// expert id, its weights are the expert's host blob); the last block publishes the work-item counts.
__global__ __launch_bounds__(kThreads) void miss_group_kernel(const int32_t* __restrict__ m_idx,
                                                             const int32_t* __restrict__ m_tok,
                                                             const int32_t* __restrict__ m_count, int n_experts,
                                                             const int32_t* __restrict__ miss_hist,
                                                             int32_t* __restrict__ row_token,
                                                             int32_t* __restrict__ pair_row, Task* __restrict__ tasks,
                                                             Task* __restrict__ big_tasks, int32_t* __restrict__ n_tasks,
                                                             int max_big, int big_ftiles, int big_rows) {
    __shared__ int lds4[kThreads / 64];
    const int e = blockIdx.x, tid = threadIdx.x;
    int all_big = 0;
    for (int q = tid; q < n_experts; q += kThreads) all_big += n_big_items(miss_hist[q], true, big_rows);
    const bool use_big = max_big > 0 && block_sum(all_big, lds4) * big_ftiles >= kMinBigUnits;
    const int upto = e < n_experts ? e : n_experts;
    int rows_before = 0, tasks_before = 0, big_before = 0;
    for (int q = tid; q < upto; q += kThreads) {
        const int m = miss_hist[q];
        rows_before += m;
        tasks_before += n_small_items(m, use_big);
        big_before += n_big_items(m, use_big, big_rows);
    }
    rows_before = block_sum(rows_before, lds4);
    tasks_before = block_sum(tasks_before, lds4);
    big_before = block_sum(big_before, lds4);
    if (e == n_experts) {
        if (tid == 0) {
            n_tasks[0] = tasks_before;
            n_tasks[1] = min(big_before, max_big);
        }
        return;
    }
    const int m = miss_hist[e];
    if (m == 0) return;
    // the miss pass reads the host's bf16 blobs
    emit_tasks(e, rows_before, m, use_big, tasks + tasks_before, big_tasks + big_before, max_big - big_before, 0, big_rows);
    collect_rows<true>(m_idx, m_tok, *m_count, 1, e, rows_before, row_token, pair_row, lds4);
}

// out[n] += sum over the token's misses, in list order, of weight * y[row]; the list is sorted by token,
// so a token's misses are one contiguous range found by bisection.  grid = (ceil(d/1024), n_tokens).
__global__ __launch_bounds__(256) void miss_combine_kernel(const float* __restrict__ y, const int32_t* __restrict__ m_idx,
                                                           const int32_t* __restrict__ m_tok,
                                                           const float* __restrict__ m_w,
                                                           const int32_t* __restrict__ pair_row,
                                                           const int32_t* __restrict__ m_count, int d,
                                                           float* __restrict__ out) {
    const int n = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    const int total = *m_count;
    int lo = 0, hi = total;                                  // first entry with token >= n
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (m_tok[mid] < n) lo = mid + 1; else hi = mid;
    }
    float4 acc = *reinterpret_cast<const float4*>(out + (int64_t)n * d + c);
    bool any = false;
    for (int p = lo; p < total && m_tok[p] == n; ++p) {
        if (m_idx[p] < 0) continue;
        const float w = m_w[p];
        const float4 v = *reinterpret_cast<const float4*>(y + (int64_t)pair_row[p] * d + c);
        acc.x = fmaf(w, v.x, acc.x);
        acc.y = fmaf(w, v.y, acc.y);
        acc.z = fmaf(w, v.z, acc.z);
        acc.w = fmaf(w, v.w, acc.w);
        any = true;
    }
    if (any) *reinterpret_cast<float4*>(out + (int64_t)n * d + c) = acc;
}

// Hands a step's miss list to the host: the first min(*n_miss, cap) entries, their number, and the token states
// (bf16 rows of d elements) of the tokens that appear in them, written straight into pinned host memory.  Four list
// entries per block; a token's row is copied by the block that holds the first entry of the token's run (the list is
// ordered by token; a row copied twice because of an unordered list is the same row).
__global__ __launch_bounds__(256) void miss_export_kernel(const tide_miss* __restrict__ miss, int cap,
                                                          const int32_t* __restrict__ n_miss,
                                                          const uint16_t* __restrict__ x, int n_tokens, int d,
                                                          tide_miss* __restrict__ miss_host, int32_t* __restrict__ n_host,
                                                          uint16_t* __restrict__ x_host) {
    const int n = min(max(*n_miss, 0), cap);
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_host = n;
    const int i0 = blockIdx.x * 4;
    for (int j = 0; j < 4; ++j) {
        const int i = i0 + j;
        if (i >= n) return;
        const tide_miss m = miss[i];
        if (threadIdx.x == 0) miss_host[i] = m;
        if (m.token < 0 || m.token >= n_tokens) continue;                 // the host refuses such a list
        if (i > 0 && miss[i - 1].token == m.token) continue;
        const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)m.token * d);
        uint4* dst = reinterpret_cast<uint4*>(x_host + (int64_t)m.token * d);
        for (int c = threadIdx.x; c < d / 8; c += 256) dst[c] = src[c];
    }
}

}  // namespace

hipError_t launch_miss_export(const tide_miss* miss, int cap, const int32_t* n_miss, const uint16_t* x, int n_tokens,
                              int d, tide_miss* miss_host, int32_t* n_host, uint16_t* x_host, hipStream_t stream) {
    hipLaunchKernelGGL(miss_export_kernel, dim3(cap > 0 ? (cap + 3) / 4 : 1), dim3(256), 0, stream, miss, cap, n_miss, x,
                       n_tokens, d, miss_host, n_host, x_host);
    return hipGetLastError();
}

hipError_t launch_miss_group(const Shape& s, const Workspace& w, const tide_miss* miss, int miss_cap,
                             const int32_t* n_miss, int n_tokens, int max_big, hipStream_t stream,
                             const uint8_t* expert_mask) {
    if (miss_cap <= 0) return hipSuccess;
    hipLaunchKernelGGL(miss_prepare_kernel, dim3((miss_cap + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, miss,
                       miss_cap, n_miss, s.E, n_tokens, expert_mask, w.m_idx, w.m_tok, w.m_w, w.miss_hist, w.m_count);
    hipLaunchKernelGGL(miss_group_kernel, dim3(s.E + 1), dim3(kThreads), 0, stream, w.m_idx, w.m_tok, w.m_count, s.E,
                       w.miss_hist, w.row_token, w.pair_row, w.tasks, w.big_tasks, w.n_tasks, max_big, (s.I + 127) / 128, s.big_rows);
    return hipGetLastError();
}

hipError_t launch_miss_combine(const Shape& s, const Workspace& w, int n_tokens, float* out, hipStream_t stream) {
    hipLaunchKernelGGL(miss_combine_kernel, dim3((s.d + 1023) / 1024, n_tokens), dim3(256), 0, stream, w.y, w.m_idx,
                       w.m_tok, w.m_w, w.pair_row, w.m_count, s.d, out);
    return hipGetLastError();
}

hipError_t launch_dispatch(const Shape& s, const LayerTables& t, const Workspace& w, const int32_t* topk_idx,
                           const float* topk_w, int n_tokens, tide_miss* miss, int miss_cap, int32_t* n_miss,
                           hipStream_t stream, LaunchEvents ev) {
    TIDE_LAUNCH(dispatch_kernel, dim3(s.capacity + 2), dim3(kThreads), stream, ev, topk_idx, topk_w,
                       n_tokens, s.k, s.capacity, s.n_shared, s.E, t.slot_of, t.expert_in_slot, t.expert_p12, w.hist_step, t.hits,
                       w.row_token, w.pair_row, w.slot_off, w.tasks, w.big_tasks, w.n_tasks, miss, miss_cap, n_miss, w.counters,
                max_big_tasks_for(s, n_tokens), (s.I + 127) / 128, s.big_rows);
    return hipGetLastError();
}

}  // namespace tide
