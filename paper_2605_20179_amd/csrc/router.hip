// Router: fp32 logits, gate, in-register top-k with wavefront shuffles, and the
// per-step / per-interval hit counts (Sec. 3.1: k of E experts per token;
// Fig. 1 caption: hits = number of tokens each expert has processed).
#include "tide_internal.h"

namespace tide {

namespace {

constexpr int kTokPerWave = 8;

__device__ inline float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// One wave per (expert, group of 8 tokens): the router row is read once per group,
// each lane owns 4 consecutive columns per 256-column stripe.
__global__ __launch_bounds__(64) void router_logits_kernel(const uint16_t* __restrict__ x, int n_tokens, int d,
                                                           int n_experts, const float* __restrict__ w_r,
                                                           float* __restrict__ logits,
                                                           int32_t* __restrict__ hist_step_to_clear) {
    const int e = blockIdx.x;
    const int n0 = blockIdx.y * kTokPerWave;
    const int lane = threadIdx.x;
    if (blockIdx.x == 0 && blockIdx.y == 0 && hist_step_to_clear != nullptr) {
        for (int i = lane; i < n_experts; i += 64) hist_step_to_clear[i] = 0;
    }
    float acc[kTokPerWave];
#pragma unroll
    for (int t = 0; t < kTokPerWave; ++t) acc[t] = 0.f;
    const float* wrow = w_r + (int64_t)e * d;
    for (int j = lane * 4; j < d; j += 256) {
        const float4 wv = *reinterpret_cast<const float4*>(wrow + j);
#pragma unroll
        for (int t = 0; t < kTokPerWave; ++t) {
            const int n = n0 + t;
            if (n < n_tokens) {
                const uint2 xv = *reinterpret_cast<const uint2*>(x + (int64_t)n * d + j);
                acc[t] = fmaf(bf16_bits_to_float(xv.x & 0xFFFFu), wv.x, acc[t]);
                acc[t] = fmaf(bf16_bits_to_float(xv.x >> 16), wv.y, acc[t]);
                acc[t] = fmaf(bf16_bits_to_float(xv.y & 0xFFFFu), wv.z, acc[t]);
                acc[t] = fmaf(bf16_bits_to_float(xv.y >> 16), wv.w, acc[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < kTokPerWave; ++t) {
        float v = acc[t];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0 && n0 + t < n_tokens) logits[(int64_t)(n0 + t) * n_experts + e] = v;
    }
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// One wave per token.  Lane l holds the scores of experts l, l+64, ...; each of the k
// rounds takes the wave-wide maximum (equal values: lower expert id) and retires it.
template <int V>
__global__ __launch_bounds__(64) void topk_gate_kernel(const float* __restrict__ logits,
                                                       const float* __restrict__ bias, int n_experts, int k,
                                                       int gating, int bias_mode, int32_t* __restrict__ topk_idx,
                                                       float* __restrict__ topk_w, int32_t* __restrict__ hist_step,
                                                       int32_t* __restrict__ hits, int32_t* __restrict__ idx_copy,
                                                       float* __restrict__ w_copy) {
    const int n = blockIdx.x;
    const int lane = threadIdx.x;
    const float NEG = -__builtin_huge_valf();
    float z[V], key[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int e = j * 64 + lane;
        float v = NEG;
        if (e < n_experts) {
            v = logits[(int64_t)n * n_experts + e];
            if (bias_mode == TIDE_BIAS_LOGIT) v += bias[e];
        }
        z[j] = v;
        key[j] = v;      // both gates are monotone in the logit: select on it directly
    }
    if (bias_mode == TIDE_BIAS_SELECT) {
        // selection score = gate score + bias
        float m = NEG;
#pragma unroll
        for (int j = 0; j < V; ++j) m = fmaxf(m, z[j]);
        m = wave_max(m);
        float p[V], sum = 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int e = j * 64 + lane;
            p[j] = 0.f;
            if (e < n_experts) {
                p[j] = (gating == TIDE_GATING_SOFTMAX) ? expf(z[j] - m) : 1.f / (1.f + expf(-z[j]));
                sum += p[j];
            }
        }
        sum = wave_sum(sum);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int e = j * 64 + lane;
            if (e < n_experts) key[j] = ((gating == TIDE_GATING_SOFTMAX) ? p[j] / sum : p[j]) + bias[e];
        }
    }

    int my_e = -1;      // lane i < k keeps the i-th selection
    float my_z = 0.f;
    for (int i = 0; i < k; ++i) {
        float best = NEG;
        int be = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int e = j * 64 + lane;
            if (e < n_experts && key[j] > best) { best = key[j]; be = e; }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float ob = __shfl_xor(best, off);
            const int oe = __shfl_xor(be, off);
            if (ob > best || (ob == best && oe < be)) { best = ob; be = oe; }
        }
        if (be == 0x7fffffff) be = 0;     // only with non-finite logits; keeps indexing in range
        float zown = 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            if (j == (be >> 6)) {
                zown = z[j];
                if (lane == (be & 63)) key[j] = NEG;
            }
        }
        const float zsel = __shfl(zown, be & 63);
        if (lane == i) { my_e = be; my_z = zsel; }
    }

    float s = 0.f;
    if (gating == TIDE_GATING_SOFTMAX) {
        const float m = wave_max(lane < k ? my_z : NEG);
        if (lane < k) s = expf(my_z - m);
    } else {
        if (lane < k) s = 1.f / (1.f + expf(-my_z));
    }
    const float tot = wave_sum(s);
    if (lane < k) {
        const float w = s / tot;
        topk_idx[(int64_t)n * k + lane] = my_e;
        topk_w[(int64_t)n * k + lane] = w;
        if (idx_copy) idx_copy[(int64_t)n * k + lane] = my_e;
        if (w_copy) w_copy[(int64_t)n * k + lane] = w;
        atomicAdd(&hist_step[my_e], 1);
        atomicAdd(&hits[my_e], 1);
    }
}

__global__ void clear_i32_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ void count_pairs_kernel(const int32_t* __restrict__ topk_idx, int n_pairs, int n_experts,
                                   int32_t* hist_step, int32_t* hits) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n_pairs) {
        const int e = topk_idx[p];
        if (e < 0 || e >= n_experts) return;
        atomicAdd(&hist_step[e], 1);
        atomicAdd(&hits[e], 1);
    }
}

}  // namespace

hipError_t launch_router_logits(const Shape& s, const uint16_t* x, int n_tokens, const float* w_r, float* logits,
                                int32_t* hist_step_to_clear, hipStream_t stream) {
    dim3 grid(s.E, (n_tokens + kTokPerWave - 1) / kTokPerWave);
    hipLaunchKernelGGL(router_logits_kernel, grid, dim3(64), 0, stream, x, n_tokens, s.d, s.E, w_r, logits,
                       hist_step_to_clear);
    return hipGetLastError();
}

hipError_t launch_topk_gate(const Shape& s, const float* logits, const float* bias, int n_tokens,
                            int32_t* topk_idx, float* topk_w, int32_t* hist_step, int32_t* hits,
                            int32_t* idx_copy, float* w_copy, hipStream_t stream) {
    if (s.E <= 256) {
        hipLaunchKernelGGL(topk_gate_kernel<4>, dim3(n_tokens), dim3(64), 0, stream, logits, bias, s.E, s.k,
                           s.gating, s.bias_mode, topk_idx, topk_w, hist_step, hits, idx_copy, w_copy);
    } else {
        hipLaunchKernelGGL(topk_gate_kernel<8>, dim3(n_tokens), dim3(64), 0, stream, logits, bias, s.E, s.k,
                           s.gating, s.bias_mode, topk_idx, topk_w, hist_step, hits, idx_copy, w_copy);
    }
    return hipGetLastError();
}

hipError_t launch_clear_i32(int32_t* p, int n, hipStream_t stream) {
    hipLaunchKernelGGL(clear_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
    return hipGetLastError();
}

hipError_t launch_count_pairs(const Shape& s, const int32_t* topk_idx, int n_tokens, int32_t* hist_step,
                              int32_t* hits, hipStream_t stream) {
    hipLaunchKernelGGL(clear_i32_kernel, dim3((s.E + 255) / 256), dim3(256), 0, stream, hist_step, s.E);
    const int n_pairs = n_tokens * s.k;
    hipLaunchKernelGGL(count_pairs_kernel, dim3((n_pairs + 255) / 256), dim3(256), 0, stream, topk_idx, n_pairs,
                       s.E, hist_step, hits);
    return hipGetLastError();
}

}  // namespace tide
