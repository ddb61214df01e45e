// Weighted combine back to token order (Sec. 3.3: partial results are brought together
// at the end of the FFN block).  A per-token gather in fixed rank order -- no float
// atomics, so the output is bit-identical from run to run.
#include "tide_internal.h"

namespace tide {

namespace {

// grid = (ceil(d / 1024), n_tokens); each thread owns 4 consecutive output columns.
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ y, const int32_t* __restrict__ pair_row,
                                                      const float* __restrict__ topk_w,
                                                      const int32_t* __restrict__ slot_off, int capacity,
                                                      int n_shared, int k, int d, float* __restrict__ out) {
    const int n = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n_shared) {
        const int64_t row = (int64_t)slot_off[capacity] + n;
        acc = *reinterpret_cast<const float4*>(y + row * d + c);
    }
    for (int i = 0; i < k; ++i) {
        const int row = pair_row[(int64_t)n * k + i];
        if (row >= 0) {
            const float w = topk_w[(int64_t)n * k + i];
            const float4 v = *reinterpret_cast<const float4*>(y + (int64_t)row * d + c);
            acc.x = fmaf(w, v.x, acc.x);
            acc.y = fmaf(w, v.y, acc.y);
            acc.z = fmaf(w, v.z, acc.z);
            acc.w = fmaf(w, v.w, acc.w);
        }
    }
    *reinterpret_cast<float4*>(out + (int64_t)n * d + c) = acc;
}

// out[tokens[r]][:] += rows[r][:].  grid = (n_rows, ceil(d / 1024)).  `rows` and `tokens` may lie in pinned host
// memory: each element is read once.
__global__ __launch_bounds__(256) void add_rows_kernel(const float* __restrict__ rows, const int32_t* __restrict__ tokens,
                                                       int d, float* __restrict__ out) {
    const int r = blockIdx.x;
    const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    const float4 v = *reinterpret_cast<const float4*>(rows + (int64_t)r * d + c);
    float4* o = reinterpret_cast<float4*>(out + (int64_t)tokens[r] * d + c);
    float4 a = *o;
    a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    *o = a;
}

}  // namespace

hipError_t launch_add_rows(const float* rows, const int32_t* tokens, int n_rows, int d, float* out, hipStream_t stream) {
    if (n_rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(add_rows_kernel, dim3(n_rows, (d + 1023) / 1024), dim3(256), 0, stream, rows, tokens, d, out);
    return hipGetLastError();
}

hipError_t launch_combine(const Shape& s, const Workspace& w, const float* topk_w, int n_tokens, float* out,
                          hipStream_t stream, LaunchEvents ev) {
    dim3 grid((s.d + 1023) / 1024, n_tokens);
    TIDE_LAUNCH(combine_kernel, grid, dim3(256), stream, ev, w.y, w.pair_row, topk_w, w.slot_off, s.capacity,
                       s.n_shared, s.k, s.d, out);
    return hipGetLastError();
}

}  // namespace tide
