// Refresh step: the resident set becomes the current top-B experts by hit count
// (Alg. 1 refresh step: most-hit CPU experts in, least-hit GPU experts out; Sec. 3.3).
// One workgroup, one expert per thread, all-pairs ranking (E <= 512).
#include "packed12_device.h"
#include "tide_internal.h"

namespace tide {

namespace {

constexpr int kThreads = kMaxExperts;

// Orders are expressed as packed 64-bit keys so that each all-pairs pass is one LDS read
// and one compare per candidate:
//   placement rank (larger key first):  hits | resident bit | reversed id
//   leaving order  (smaller key first): hits | id
//   entering order (larger key first):  hits | reversed id
__global__ __launch_bounds__(kThreads) void refresh_select_kernel(int n_experts, int n_slots, int capacity,
                                                                  const int32_t* __restrict__ counts,
                                                                  int32_t* __restrict__ hits_to_reset,
                                                                  int32_t* __restrict__ slot_of,
                                                                  int32_t* __restrict__ expert_in_slot,
                                                                  RefreshOut* __restrict__ out) {
    __shared__ unsigned long long rank_key[kMaxExperts];
    __shared__ unsigned long long leave_key[kMaxExperts];   // ~0 for experts that are not leaving
    __shared__ unsigned long long enter_key[kMaxExperts];   // 0 for experts that are not entering
    __shared__ int free_slot[kMaxExperts];   // freed slots in leaving order, then empty slots ascending
    __shared__ int plan_expert[kMaxExperts], plan_slot[kMaxExperts];
    __shared__ int empty_flag[kMaxExperts];
    __shared__ int n_leaving_s, n_entering_s;
    const int e = threadIdx.x;
    const bool live = e < n_experts;
    unsigned long long h = 0;
    int my_slot = -1;
    if (live) {
        h = (unsigned long long)(unsigned int)counts[e];
        my_slot = slot_of[e];
    }
    rank_key[e] = live ? ((h << 10) | (my_slot >= 0 ? 512ull : 0ull) | (unsigned long long)(kMaxExperts - 1 - e)) : 0ull;
    empty_flag[e] = (e < n_slots && expert_in_slot[e] < 0) ? 1 : 0;
    if (e == 0) { n_leaving_s = 0; n_entering_s = 0; }
    __syncthreads();

    int my_cls = 0;            // 1 leaving, 2 entering
    if (live) {
        const unsigned long long mine = rank_key[e];
        int rank = 0;
#pragma unroll 8
        for (int o = 0; o < n_experts; ++o) rank += rank_key[o] > mine ? 1 : 0;
        const bool in_new = rank < capacity;
        if (my_slot >= 0 && !in_new) my_cls = 1;
        if (my_slot < 0 && in_new) my_cls = 2;
    }
    leave_key[e] = my_cls == 1 ? ((h << 10) | (unsigned long long)e) : ~0ull;
    enter_key[e] = my_cls == 2 ? ((h << 10) | (unsigned long long)(kMaxExperts - 1 - e) | (1ull << 62)) : 0ull;
    if (my_cls == 1) atomicAdd(&n_leaving_s, 1);
    if (my_cls == 2) atomicAdd(&n_entering_s, 1);
    __syncthreads();
    const int n_leaving = n_leaving_s, n_entering = n_entering_s;

    int my_pos = -1;
    if (my_cls == 1) {
        const unsigned long long mine = leave_key[e];
        int pos = 0;
#pragma unroll 8
        for (int o = 0; o < n_experts; ++o) pos += leave_key[o] < mine ? 1 : 0;
        my_pos = pos;
        free_slot[pos] = my_slot;
    } else if (my_cls == 2) {
        const unsigned long long mine = enter_key[e];
        int pos = 0;
#pragma unroll 8
        for (int o = 0; o < n_experts; ++o) pos += enter_key[o] > mine ? 1 : 0;
        my_pos = pos;
    }
    // thread s < n_slots looks at slot s: originally empty slots follow the freed ones
    if (e < n_slots && empty_flag[e]) {
        int before = 0;
        for (int q = 0; q < e; ++q) before += empty_flag[q];
        free_slot[n_leaving + before] = e;
    }
    __syncthreads();

    if (my_cls == 1) {
        expert_in_slot[my_slot] = -1;
        slot_of[e] = -1;
    }
    __syncthreads();
    if (my_cls == 2) {
        const int s = free_slot[my_pos];
        expert_in_slot[s] = e;
        slot_of[e] = s;
        plan_expert[my_pos] = e;
        plan_slot[my_pos] = s;
    }
    if (live && hits_to_reset != nullptr) hits_to_reset[e] = 0;
    __syncthreads();
    // results go to host-visible memory in thread order (coalesced stores)
    if (e < n_entering) {
        out->expert[e] = plan_expert[e];
        out->slot[e] = plan_slot[e];
    }
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

namespace {
// The refresh's host-to-device copies as one kernel: the newcomers' blobs are read in place from pinned
// host memory (the plan itself is read from the pinned block the selection kernel wrote) and stored to
// their cache slots -- or, for a deferred refresh, to staging blob i.  Sixteen workgroups keep the host link
// busy (56.9 GB/s against 52.7 GB/s for one DMA per 6 MiB blob); more would not copy faster, and every compute
// unit that hosts one serves the step kernels' own loads slowly while the copy lasts (its vector memory
// pipeline is full of host-link reads).  Each thread keeps four 16-byte reads in flight.
constexpr int kCopyBlocks = 16, kCopyThreads = 256;
// n16 16-byte pieces from src to dst, spread over the launch; each thread keeps four reads in flight
__device__ inline void copy_blob(const uint8_t* src_bytes, uint8_t* dst_bytes, uint64_t n16) {
    const uint4* src = reinterpret_cast<const uint4*>(src_bytes);
    uint4* dst = reinterpret_cast<uint4*>(dst_bytes);
    const uint64_t stride = (uint64_t)gridDim.x * kCopyThreads;
    uint64_t q = (uint64_t)blockIdx.x * kCopyThreads + threadIdx.x;
    for (; q + 3 * stride < n16; q += 4 * stride) {
        const uint4 a = src[q], b = src[q + stride], c = src[q + 2 * stride], d = src[q + 3 * stride];
        dst[q] = a;
        dst[q + stride] = b;
        dst[q + 2 * stride] = c;
        dst[q + 3 * stride] = d;
    }
    for (; q < n16; q += stride) dst[q] = src[q];
}

__global__ __launch_bounds__(kCopyThreads) void refresh_copy_kernel(const uint8_t* __restrict__ host_blobs, uint64_t host_stride,
                                                                   uint64_t blob_bytes, uint8_t* __restrict__ dst_base,
                                                                   const RefreshOut* __restrict__ plan, int n, int dst_by_rank) {
    if (n < 0) n = plan->n_copies;             // queued without the host knowing the plan
    for (int i = 0; i < n; ++i)
        copy_blob(host_blobs + (uint64_t)plan->expert[i] * host_stride,
                  dst_base + (uint64_t)(dst_by_rank ? i : plan->slot[i]) * blob_bytes, blob_bytes / 16);
}

// The same copies from the 12-bit form of the blobs (packed12.h): 3/4 of the bytes cross the host link.
//   verbatim: the slots keep the 12-bit form (the expert GEMMs decode it): the compressed blob is copied as it is.
//   else:     a wave decodes one tile per turn -- lane l reads its 3 dwords at byte 12 l of the tile's payload and the
//             tile's 16-byte table, and writes its 8 bf16 (16 bytes) -- and keeps six tiles in flight.
// An expert whose header says "raw" is copied from the raw blob either way.
constexpr int kP12InFlight = 6;      // tiles a wave has in flight: 72 bytes per lane, as many as the raw copy's 64
__global__ __launch_bounds__(kCopyThreads) void refresh_copy_p12_kernel(const uint8_t* __restrict__ comp_blobs, uint64_t comp_stride,
                                                                       const uint8_t* __restrict__ host_blobs, uint64_t host_stride,
                                                                       uint64_t blob_bytes, uint8_t* __restrict__ dst_base,
                                                                       const RefreshOut* __restrict__ plan, int n, int dst_by_rank,
                                                                       int verbatim, int d, int d_ff) {
    const int lane = threadIdx.x & 63;
    const uint32_t wave = (blockIdx.x * kCopyThreads + threadIdx.x) >> 6, n_waves = gridDim.x * (kCopyThreads / 64);
    const uint32_t n_tiles = (uint32_t)(blob_bytes / 1024);
    const P12Layout lay = p12_layout(n_tiles);
    if (n < 0) n = plan->n_copies;             // queued without the host knowing the plan
    for (int i = 0; i < n; ++i) {
        const uint8_t* comp = comp_blobs + (uint64_t)plan->expert[i] * comp_stride;
        uint8_t* dst = dst_base + (uint64_t)(dst_by_rank ? i : plan->slot[i]) * blob_bytes;
        if (reinterpret_cast<const P12Header*>(comp)->raw) {
            copy_blob(host_blobs + (uint64_t)plan->expert[i] * host_stride, dst, blob_bytes / 16);
            continue;
        }
        if (verbatim) {
            copy_blob(comp, dst, lay.bytes / 16);
            continue;
        }
        const uint8_t* table = comp + lay.off_table;
        const uint8_t* payload = comp + lay.off_payload + lane * 12;
        uint32_t t = wave;
        for (; t + (kP12InFlight - 1) * n_waves < n_tiles; t += kP12InFlight * n_waves) {
            P12Words w[kP12InFlight];
            uint4 tab[kP12InFlight];
#pragma unroll
            for (int u = 0; u < kP12InFlight; ++u) {
                w[u] = *reinterpret_cast<const P12Words*>(payload + (uint64_t)(t + u * n_waves) * kP12TileBytes);
                tab[u] = *reinterpret_cast<const uint4*>(table + (uint64_t)p12_table_slot(t + u * n_waves, d, d_ff) * kP12TableBytes);
            }
#pragma unroll
            for (int u = 0; u < kP12InFlight; ++u)
                *reinterpret_cast<uint4*>(dst + (uint64_t)(t + u * n_waves) * 1024 + lane * 16) = p12_decode(w[u], tab[u]);
        }
        for (; t < n_tiles; t += n_waves)
            *reinterpret_cast<uint4*>(dst + (uint64_t)t * 1024 + lane * 16) =
                p12_decode(*reinterpret_cast<const P12Words*>(payload + (uint64_t)t * kP12TileBytes),
                           *reinterpret_cast<const uint4*>(table + (uint64_t)p12_table_slot(t, d, d_ff) * kP12TableBytes));
    }
}

// Measurement only: every workgroup reads its share of `bytes` once, front to back, with the access shape of the
// expert GEMMs' weight stream -- each wave fetches whole 1 KiB tiles, 16 bytes per lane, non-temporal, eight tiles
// in flight -- and folds what it read into one word per thread so that the loads cannot be dropped.
constexpr int kProbeInFlight = 8;
__global__ __launch_bounds__(256) void stream_probe_kernel(const uint8_t* __restrict__ base, uint64_t tiles, uint32_t* __restrict__ sink) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t wave = ((uint64_t)blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = (uint64_t)gridDim.x * 4;
    // a wave owns a contiguous run of tiles (as a GEMM workgroup walks one contiguous region)
    const uint64_t per = (tiles + n_waves - 1) / n_waves;
    const uint64_t t0 = wave * per, t1 = t0 + per < tiles ? t0 + per : tiles;
    uint32_t acc = 0;
    uint64_t t = t0;
    for (; t + kProbeInFlight <= t1; t += kProbeInFlight) {
        u32x4 v[kProbeInFlight];
#pragma unroll
        for (int u = 0; u < kProbeInFlight; ++u)
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (t + u) * 1024 + lane * 16));
#pragma unroll
        for (int u = 0; u < kProbeInFlight; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; t < t1; ++t) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + t * 1024 + lane * 16));
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;          // practically never true: the store only keeps the reads alive
}

__global__ void scale_counts_kernel(int32_t* hits, int n, int num, int den) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n) hits[e] = (int32_t)(((int64_t)hits[e] * num) / den);
}
}  // namespace

// A copy workgroup asks for almost all of a compute unit's LDS without using it: no workgroup of the expert GEMM
// kernels (which stage their token rows in LDS) then fits beside it, so the copy's host-link reads never sit in the
// memory pipeline of a compute unit that a GEMM workgroup is waiting on.
constexpr int kCopyLdsReserve = 152 * 1024;
template <typename K>
hipError_t reserve_lds(K kernel) {
    static hipError_t rc = kCopyLdsReserve > 0 ? hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kCopyLdsReserve)
                                               : hipSuccess;
    return rc;
}

hipError_t launch_refresh_copies(const uint8_t* host_blobs, uint64_t host_stride, uint64_t blob_bytes, uint8_t* dst_base,
                                 const RefreshOut* plan, int n, bool dst_by_rank, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (hipError_t rc = reserve_lds(refresh_copy_kernel); rc != hipSuccess) return rc;
    hipLaunchKernelGGL(refresh_copy_kernel, dim3(kCopyBlocks), dim3(kCopyThreads), kCopyLdsReserve, stream, host_blobs, host_stride,
                       blob_bytes, dst_base, plan, n, dst_by_rank ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_refresh_copies_p12(const uint8_t* comp_blobs, uint64_t comp_stride, const uint8_t* host_blobs,
                                     uint64_t host_stride, uint64_t blob_bytes, uint8_t* dst_base, const RefreshOut* plan, int n,
                                     bool dst_by_rank, bool verbatim, int d, int d_ff, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (hipError_t rc = reserve_lds(refresh_copy_p12_kernel); rc != hipSuccess) return rc;
    hipLaunchKernelGGL(refresh_copy_p12_kernel, dim3(kCopyBlocks), dim3(kCopyThreads), kCopyLdsReserve, stream, comp_blobs, comp_stride,
                       host_blobs, host_stride, blob_bytes, dst_base, plan, n, dst_by_rank ? 1 : 0, verbatim ? 1 : 0, d, d_ff);
    return hipGetLastError();
}

hipError_t launch_stream_probe(const uint8_t* base, uint64_t bytes, int workgroups, uint32_t* sink, hipStream_t stream, LaunchEvents ev) {
    TIDE_LAUNCH(stream_probe_kernel, dim3(workgroups), dim3(256), stream, ev, base, bytes / 1024, sink);
    return hipGetLastError();
}

hipError_t launch_scale_counts(int32_t* hits, int n_experts, int num, int den, hipStream_t stream) {
    hipLaunchKernelGGL(scale_counts_kernel, dim3((n_experts + 255) / 256), dim3(256), 0, stream, hits, n_experts, num, den);
    return hipGetLastError();
}

}  // namespace tide
