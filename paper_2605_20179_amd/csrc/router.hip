// Router: fp32-faithful logits on the bf16 matrix cores, gate, in-register top-k with
// wavefront shuffles, and the
// per-step / per-interval hit counts (Sec. 3.1: k of E experts per token;
// Fig. 1 caption: hits = number of tokens each expert has processed).
#include "dispatch_small.h"
#include "tide_internal.h"

#include <type_traits>

namespace tide {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kRouterWaves = 4;

// An fp32 number is the exact sum of three bf16 numbers (its mantissa cut into 8-bit
// pieces); the hidden states are bf16 already.  So the fp32 router product
// x * w = x*hi + x*mid + x*lo runs on the bf16 matrix cores with every product exact in
// fp32 and only the accumulation rounded -- the same error class as an fp32 FMA chain.
__device__ inline void split3(float w, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    const uint32_t wb = __float_as_uint(w);
    hi = wb & 0xFFFF0000u;
    const float r1 = w - __uint_as_float(hi);
    mid = __float_as_uint(r1) & 0xFFFF0000u;
    const float r2 = r1 - __uint_as_float(mid);
    lo = __float_as_uint(r2) & 0xFFFF0000u;
}

__device__ inline bf16x8 pack8(const uint32_t (&v)[8]) {
    u32x4 p;
    p[0] = (v[0] >> 16) | v[1];
    p[1] = (v[2] >> 16) | v[3];
    p[2] = (v[4] >> 16) | v[5];
    p[3] = (v[6] >> 16) | v[7];
    return __builtin_bit_cast(bf16x8, p);
}

// z_part[ks][n][e] = sum over the ks-th slice of the hidden dimension of x[n][j] * W_r[e][j].
// grid.x = expert tile (16 experts) * k_splits + ks, grid.y = token tile (NT*16 tokens);
// the 4 waves of a workgroup interleave over the slice's 32-column chunks and are summed
// through LDS in a fixed order.  MFMA layout: experts on the 16-row side, tokens on the
// 16-column side.
template <int NT>
__global__ __launch_bounds__(kRouterWaves * 64) void router_logits_kernel(
    const uint16_t* __restrict__ x, int n_tokens, int d, int n_experts, int e_pad, int k_splits,
    const float* __restrict__ w_r, float* __restrict__ z_part, int32_t* __restrict__ hist_step_to_clear) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int etile = blockIdx.x / k_splits, ks = blockIdx.x % k_splits;
    const int n0 = blockIdx.y * (NT * 16);
    if (blockIdx.x == 0 && blockIdx.y == 0 && hist_step_to_clear != nullptr) {
        for (int i = threadIdx.x; i < n_experts; i += kRouterWaves * 64) hist_step_to_clear[i] = 0;
    }
    const int chunks_per_split = (d >> 5) / k_splits;
    const int c_begin = ks * chunks_per_split, c_end = c_begin + chunks_per_split;
    const int erow = min(etile * 16 + (lane & 15), n_experts - 1);           // clamp: padded rows are never stored
    const float* wrow = w_r + (int64_t)erow * d + (lane >> 4) * 8;
    const uint16_t* xrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = min(n0 + t * 16 + (lane & 15), n_tokens - 1);
        xrow[t] = x + (int64_t)n * d + (lane >> 4) * 8;
    }
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int c = c_begin + wave; c < c_end; c += kRouterWaves) {
        const float4 w0 = *reinterpret_cast<const float4*>(wrow + c * 32);
        const float4 w1 = *reinterpret_cast<const float4*>(wrow + c * 32 + 4);
        bf16x8 b[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) b[t] = *reinterpret_cast<const bf16x8*>(xrow[t] + c * 32);
        const float wv[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
        uint32_t hi[8], mid[8], lo[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) split3(wv[i], hi[i], mid[i], lo[i]);
        const bf16x8 a_hi = pack8(hi), a_mid = pack8(mid), a_lo = pack8(lo);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, b[t], acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_mid, b[t], acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, b[t], acc[t], 0, 0, 0);
        }
    }
    __shared__ f32x4 red[kRouterWaves][NT][64];
#pragma unroll
    for (int t = 0; t < NT; ++t) red[wave][t][lane] = acc[t];
    __syncthreads();
    // wave w finishes token tiles w, w+4, ...
    for (int t = wave; t < NT; t += kRouterWaves) {
        const f32x4 v = red[0][t][lane] + red[1][t][lane] + red[2][t][lane] + red[3][t][lane];
        const int n = n0 + t * 16 + (lane & 15);
        const int e = etile * 16 + (lane >> 4) * 4;
        if (n < n_tokens)
            *reinterpret_cast<float4*>(z_part + ((int64_t)ks * n_tokens + n) * e_pad + e) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// The same product for steps of many tokens: a workgroup computes 64 experts (one 16-expert tile per
// wave) x 128 tokens over one slice of the hidden dimension.  The token rows are shared by the four
// waves, so they are staged through LDS, 128 columns at a time and double-buffered (one barrier per
// stage); each wave converts its own router rows.  Against the small-step kernel this cuts the L2
// traffic per flop by 4 (every x element is fetched by E/64 workgroups instead of E/16).
constexpr int kWideTokens = 128, kWideNT = kWideTokens / 16, kWideStageChunks = 4;
constexpr int kWideRowElems = kWideStageChunks * 32 + 8;      // +16 B per row: conflict-free fragment reads
__global__ __launch_bounds__(kRouterWaves * 64) void router_logits_wide_kernel(
    const uint16_t* __restrict__ x, int n_tokens, int d, int n_experts, int e_pad, int k_splits,
    const float* __restrict__ w_r, float* __restrict__ z_part, int32_t* __restrict__ hist_step_to_clear) {
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][kWideTokens * kWideRowElems];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int egroup = blockIdx.x / k_splits, ks = blockIdx.x % k_splits;
    const int n0 = blockIdx.y * kWideTokens;
    if (blockIdx.x == 0 && blockIdx.y == 0 && hist_step_to_clear != nullptr) {
        for (int i = threadIdx.x; i < n_experts; i += kRouterWaves * 64) hist_step_to_clear[i] = 0;
    }
    const int chunks_per_split = (d >> 5) / k_splits;             // a multiple of kWideStageChunks (launcher)
    const int c_begin = ks * chunks_per_split;
    const int stages = chunks_per_split / kWideStageChunks;
    const int etile = egroup * kRouterWaves + wave;
    const bool active = etile * 16 < n_experts;                   // a spare wave still stages and keeps the barriers
    const int erow = min(etile * 16 + (lane & 15), n_experts - 1);
    const float* wrow = w_r + (int64_t)erow * d + (lane >> 4) * 8 + c_begin * 32;

    // staging map: piece q = tid + 256*j is row q / 16 of the token tile, columns (q % 16)*8 .. +7 of the stage
    constexpr int kPieces = kWideTokens * kWideStageChunks * 4 / 256;
    const uint16_t* xsrc[kPieces];
#pragma unroll
    for (int j = 0; j < kPieces; ++j) {
        const int q = threadIdx.x + 256 * j;
        const int n = min(n0 + q / 16, n_tokens - 1);             // padding rows mirror the last token; never stored
        xsrc[j] = x + (int64_t)n * d + c_begin * 32 + (q % 16) * 8;
    }
    u32x4 xr[kPieces];
    auto fetch = [&](int stage) {
#pragma unroll
        for (int j = 0; j < kPieces; ++j) xr[j] = *reinterpret_cast<const u32x4*>(xsrc[j] + stage * kWideStageChunks * 32);
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int q = threadIdx.x + 256 * j;
            *reinterpret_cast<u32x4*>(&xs[buf][(q / 16) * kWideRowElems + (q % 16) * 8]) = xr[j];
        }
    };
    f32x4 acc[kWideNT];
#pragma unroll
    for (int t = 0; t < kWideNT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    fetch(0);
    store(0);
    fetch(min(1, stages - 1));
    float4 w0 = *reinterpret_cast<const float4*>(wrow), w1 = *reinterpret_cast<const float4*>(wrow + 4);
    __syncthreads();
    for (int stage = 0; stage < stages; ++stage) {
        // the other buffer was last read in stage-1, which every wave left through the barrier below
        store((stage + 1) & 1);
        fetch(min(stage + 2, stages - 1));
        const uint16_t* frag = &xs[stage & 1][(lane & 15) * kWideRowElems + (lane >> 4) * 8];
#pragma unroll
        for (int cc = 0; cc < kWideStageChunks; ++cc) {
            const int c = stage * kWideStageChunks + cc;
            const float wv[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            const int cn = min(c + 1, chunks_per_split - 1);       // next chunk's router weights, clamped
            w0 = *reinterpret_cast<const float4*>(wrow + cn * 32);
            w1 = *reinterpret_cast<const float4*>(wrow + cn * 32 + 4);
            bf16x8 b[kWideNT];
#pragma unroll
            for (int t = 0; t < kWideNT; ++t) b[t] = *reinterpret_cast<const bf16x8*>(frag + t * 16 * kWideRowElems + cc * 32);
            uint32_t hi[8], mid[8], lo[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) split3(wv[i], hi[i], mid[i], lo[i]);
            const bf16x8 a_hi = pack8(hi), a_mid = pack8(mid), a_lo = pack8(lo);
#pragma unroll
            for (int t = 0; t < kWideNT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, b[t], acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < kWideNT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_mid, b[t], acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < kWideNT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, b[t], acc[t], 0, 0, 0);
        }
        __syncthreads();
    }
    if (!active) return;
#pragma unroll
    for (int t = 0; t < kWideNT; ++t) {
        const int n = n0 + t * 16 + (lane & 15);
        const int e = etile * 16 + (lane >> 4) * 4;
        if (n < n_tokens)
            *reinterpret_cast<float4*>(z_part + ((int64_t)ks * n_tokens + n) * e_pad + e) =
                make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
    }
}

// Cross-lane moves inside a row of 16 lanes by DPP rotation (no LDS round trip).  Four
// rotate-and-combine steps (by 8, 4, 2, 1) leave every lane with the combination of all 16.
template <int N>
__device__ inline int row_ror_i(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x120 + N, 0xF, 0xF, false); }
template <int N>
__device__ inline float row_ror_f(float v) { return __int_as_float(row_ror_i<N>(__float_as_int(v))); }

__device__ inline float group16_sum(float v) {
    v += row_ror_f<8>(v);
    v += row_ror_f<4>(v);
    v += row_ror_f<2>(v);
    v += row_ror_f<1>(v);
    return v;
}
__device__ inline float group16_max(float v) {
    v = fmaxf(v, row_ror_f<8>(v));
    v = fmaxf(v, row_ror_f<4>(v));
    v = fmaxf(v, row_ror_f<2>(v));
    v = fmaxf(v, row_ror_f<1>(v));
    return v;
}
__device__ inline int group16_min(int v) {
    v = min(v, row_ror_i<8>(v));
    v = min(v, row_ror_i<4>(v));
    v = min(v, row_ror_i<2>(v));
    v = min(v, row_ror_i<1>(v));
    return v;
}

// sub-lane s owns experts s*4..s*4+3 of every group of 64, so that one 16-byte load per group and
// slice fetches them; value j of the lane is expert EXPERT_OF(j)
#define EXPERT_OF(j) ((((j) >> 2) << 6) + s * 4 + ((j) & 3))

// Logits of 16 tokens (token n_base + tid/16), summed over the KS slices in slice order, plus the
// logit bias.  Every load is unconditional and independent, so they are all in flight together:
// one memory round trip instead of one per slice.
template <int V, int KS>
__device__ inline void load_logits16(int n_base, const float* __restrict__ z_part, int e_pad,
                                     const float* __restrict__ bias, int bias_mode, int n_tokens, int n_experts,
                                     float (&z)[V]) {
    const int s = threadIdx.x & 15;
    const int n = min(n_base + (int)(threadIdx.x >> 4), n_tokens - 1);
    float4 part[KS][V / 4];
#pragma unroll
    for (int p = 0; p < KS; ++p) {
        const float* row = z_part + ((int64_t)p * n_tokens + n) * e_pad;
#pragma unroll
        for (int g = 0; g < V / 4; ++g) {
            const int col = min(g * 64 + s * 4, e_pad - 4);          // clamped: columns past E are masked below
            part[p][g] = *reinterpret_cast<const float4*>(row + col);
        }
    }
    float b[V];
    if (bias_mode == TIDE_BIAS_LOGIT) {              // one uniform branch around all the loads
#pragma unroll
        for (int j = 0; j < V; ++j) b[j] = bias[min(EXPERT_OF(j), n_experts - 1)];
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) b[j] = 0.f;
    }
#pragma unroll
    for (int g = 0; g < V / 4; ++g) {
        float4 acc = part[0][g];
#pragma unroll
        for (int p = 1; p < KS; ++p) {
            acc.x += part[p][g].x;
            acc.y += part[p][g].y;
            acc.z += part[p][g].z;
            acc.w += part[p][g].w;
        }
        z[g * 4 + 0] = acc.x + b[g * 4 + 0];
        z[g * 4 + 1] = acc.y + b[g * 4 + 1];
        z[g * 4 + 2] = acc.z + b[g * 4 + 2];
        z[g * 4 + 3] = acc.w + b[g * 4 + 3];
    }
}

template <int V>
__device__ inline void load_logits16_any(int k_splits, int n_base, const float* __restrict__ z_part, int e_pad,
                                         const float* __restrict__ bias, int bias_mode, int n_tokens, int n_experts,
                                         float (&z)[V]) {
    switch (k_splits) {
        case 1: load_logits16<V, 1>(n_base, z_part, e_pad, bias, bias_mode, n_tokens, n_experts, z); break;
        case 2: load_logits16<V, 2>(n_base, z_part, e_pad, bias, bias_mode, n_tokens, n_experts, z); break;
        case 4: load_logits16<V, 4>(n_base, z_part, e_pad, bias, bias_mode, n_tokens, n_experts, z); break;
        default: load_logits16<V, 8>(n_base, z_part, e_pad, bias, bias_mode, n_tokens, n_experts, z); break;
    }
}

// Gate, top-k and weights of the tokens whose (biased) logits are in z: one token per 16 lanes, NG tokens per
// 16-lane group (both callers use NG = 1 and fill the SIMDs with more waves instead: measured faster than two
// interleaved tokens per group).
// SMALL = true: the caller is the single workgroup that routes the whole step; selections are mirrored into LDS
// (s_idx, s_w) and recorded as per-expert token masks (s_mask); otherwise hist_step[e] is incremented per
// selection (the caller passes its workgroup's LDS counts).
template <int V, bool SMALL, int NG>
__device__ inline void select16(int n_base, float (&z)[NG][V], const float* __restrict__ bias, int n_tokens,
                                int n_experts, int k, int gating, int bias_mode, int32_t* __restrict__ topk_idx,
                                float* __restrict__ topk_w, int32_t* __restrict__ hist_step,
                                int32_t* __restrict__ idx_copy,
                                float* __restrict__ w_copy, unsigned* s_mask, int* s_idx, float* s_w) {
    const int s = threadIdx.x & 15;
    const float NEG = -__builtin_huge_valf();
    int n[NG];
    bool valid[NG];
    float key[NG][V];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int n_raw = n_base + g * 16 + (threadIdx.x >> 4);
        valid[g] = n_raw < n_tokens;
        n[g] = valid[g] ? n_raw : n_tokens - 1;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            if (EXPERT_OF(j) >= n_experts) z[g][j] = NEG;
            key[g][j] = z[g][j];      // both gates are monotone in the logit: select on it directly
        }
    }
    if (bias_mode == TIDE_BIAS_SELECT) {
        // selection score = gate score + bias
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float m = NEG;
#pragma unroll
            for (int j = 0; j < V; ++j) m = fmaxf(m, z[g][j]);
            m = group16_max(m);
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < V; ++j) {
                if (EXPERT_OF(j) < n_experts) {
                    key[g][j] = (gating == TIDE_GATING_SOFTMAX) ? expf(z[g][j] - m) : 1.f / (1.f + expf(-z[g][j]));
                    sum += key[g][j];
                }
            }
            sum = group16_sum(sum);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const int e = EXPERT_OF(j);
                if (e < n_experts) key[g][j] = ((gating == TIDE_GATING_SOFTMAX) ? key[g][j] / sum : key[g][j]) + bias[e];
            }
        }
    }

    int my_e[NG];       // sub-lane i < k keeps the i-th selection
    float my_z[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) { my_e[g] = 0; my_z[g] = 0.f; }
    // One selection round: the group's largest key (per-lane maximum, then four rotations), the lowest expert id
    // that holds it (equal keys: the lower id wins, as in a stable descending sort), removal of that one value.
    // Everything is select instructions, no branches; experts past E and values already taken hold -inf and never
    // win.  SEL: the gate needs the winner's logit, which is not its key (selection score = gate score + bias).
    auto rounds = [&](auto sel) {
        constexpr bool SEL = decltype(sel)::value;
        for (int i = 0; i < k; ++i) {
            float gmax[NG];
            int gid[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                float m = key[g][0];
#pragma unroll
                for (int j = 1; j < V; ++j) m = fmaxf(m, key[g][j]);
                gmax[g] = m;
            }
#pragma unroll
            for (int g = 0; g < NG; ++g) gmax[g] = group16_max(gmax[g]);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                int c = 0x7fffffff;
#pragma unroll
                for (int j = V - 1; j >= 0; --j) c = (key[g][j] == gmax[g]) ? EXPERT_OF(j) : c;     // ascending in j = ascending id
                gid[g] = (gmax[g] > NEG) ? c : 0x7fffffff;
            }
#pragma unroll
            for (int g = 0; g < NG; ++g) gid[g] = group16_min(gid[g]);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                float zw = NEG;
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    const bool hit = EXPERT_OF(j) == gid[g];
                    if (SEL) zw = hit ? z[g][j] : zw;
                    key[g][j] = hit ? NEG : key[g][j];
                }
                const bool none = gid[g] == 0x7fffffff;      // only with non-finite logits; keeps indexing in range
                const float bz = SEL ? group16_max(zw) : gmax[g];
                my_e[g] = (s == i) ? (none ? 0 : gid[g]) : my_e[g];
                my_z[g] = (s == i) ? (none ? 0.f : bz) : my_z[g];
            }
        }
    };
    if (bias_mode == TIDE_BIAS_SELECT) rounds(std::true_type{}); else rounds(std::false_type{});

#pragma unroll
    for (int g = 0; g < NG; ++g) {
        float sc = 0.f;
        if (gating == TIDE_GATING_SOFTMAX) {
            const float m = group16_max(s < k ? my_z[g] : NEG);
            if (s < k) sc = expf(my_z[g] - m);
        } else {
            if (s < k) sc = 1.f / (1.f + expf(-my_z[g]));
        }
        const float tot = group16_sum(sc);
        if (valid[g] && s < k) {
            const float w = sc / tot;
            const int64_t p = (int64_t)n[g] * k + s;
            topk_idx[p] = my_e[g];
            topk_w[p] = w;
            if (idx_copy) idx_copy[p] = my_e[g];
            if (w_copy) w_copy[p] = w;
            if (SMALL) {
                atomicOr(&s_mask[my_e[g]], 1u << n[g]);      // which tokens chose the expert (order-free)
                s_idx[p] = my_e[g];
                s_w[p] = w;
            } else {
                atomicAdd(&hist_step[my_e[g]], 1);    // the caller's per-workgroup counts
            }
        }
    }
}

template <int V>
__global__ __launch_bounds__(256) void topk_gate_kernel(const float* __restrict__ z_part, int k_splits, int e_pad,
                                                        const float* __restrict__ bias, int n_tokens, int n_experts,
                                                        int k, int gating, int bias_mode,
                                                        int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                        int32_t* __restrict__ hist_step,
                                                        int32_t* __restrict__ idx_copy, float* __restrict__ w_copy) {
    // the workgroup's 16 tokens are counted in LDS first: a popular expert then costs one global atomic per
    // workgroup instead of one per token (thousands on one address at thousands of tokens per step)
    __shared__ int32_t s_hist[kMaxExperts];
    for (int e = threadIdx.x; e < n_experts; e += 256) s_hist[e] = 0;
    float z[1][V];
    load_logits16_any<V>(k_splits, blockIdx.x * 16, z_part, e_pad, bias, bias_mode, n_tokens, n_experts, z[0]);
    __syncthreads();
    select16<V, false, 1>(blockIdx.x * 16, z, bias, n_tokens, n_experts, k, gating, bias_mode, topk_idx, topk_w,
                          s_hist, idx_copy, w_copy, nullptr, nullptr, nullptr);
    __syncthreads();
    for (int e = threadIdx.x; e < n_experts; e += 256) {
        const int c = s_hist[e];
        if (c) atomicAdd(&hist_step[e], c);           // H += hist_step follows in the split kernel (one writer)
    }
}

// A step of at most 32 tokens is routed by ONE workgroup: top-k of every token, the step's
// histogram (in LDS), H += histogram, then the hit/miss split -- all without leaving the CU, so
// nothing has to travel through memory between routing and split and no launch separates them.
// 16 lanes per token: the 32 tokens fill eight waves, two per SIMD, whose selection rounds (the
// kernel's longest phase, bound by vector-ALU issue) interleave.
template <int V>
__global__ __launch_bounds__(kRouteThreads) void route_small_kernel(const float* __restrict__ z_part, int k_splits, int e_pad,
                                                          const float* __restrict__ bias, int n_experts, int gating,
                                                          int bias_mode, int32_t* __restrict__ topk_idx,
                                                          float* __restrict__ topk_w, int32_t* __restrict__ hist_step,
                                                          int32_t* __restrict__ hits,
                                                          int32_t* __restrict__ idx_copy, float* __restrict__ w_copy,
                                                          DispatchArgs da) {
    static_assert(kRouteThreads == 16 * kSmallDispatchMaxTokens && kMaxExperts % kRouteThreads == 0, "one 16-lane group per token");
    __shared__ unsigned s_mask[kMaxExperts];     // per expert: bit n set when token n selected it
    __shared__ int s_slot_of[kMaxExperts];
    __shared__ int s_eis[kMaxExperts];
    __shared__ int s_idx[kSmallDispatchMaxPairs];
    __shared__ float s_w[kSmallDispatchMaxPairs];
    __shared__ int s_work[kSmallDispatchLdsInts];
    // everything the workgroup needs from memory is requested up front -- the placement tables and the
    // logits of every token -- because each dependent round trip to memory costs microseconds
    int t_slot[kMaxExperts / kRouteThreads], t_eis[kMaxExperts / kRouteThreads];
#pragma unroll
    for (int q = 0; q < kMaxExperts / kRouteThreads; ++q) {
        const int e = threadIdx.x + kRouteThreads * q;
        t_slot[q] = da.slot_of[min(e, n_experts - 1)];
        t_eis[q] = da.expert_in_slot[min(e, da.capacity - 1)];
    }
    float z[1][V];
    load_logits16_any<V>(k_splits, 0, z_part, e_pad, bias, bias_mode, da.n_tokens, n_experts, z[0]);
#pragma unroll
    for (int q = 0; q < kMaxExperts / kRouteThreads; ++q) {
        const int e = threadIdx.x + kRouteThreads * q;
        s_mask[e] = 0u;
        s_slot_of[e] = t_slot[q];
        s_eis[e] = t_eis[q];
    }
    __syncthreads();
    select16<V, true, 1>(0, z, bias, da.n_tokens, n_experts, da.k, gating, bias_mode, topk_idx, topk_w, nullptr,
                         idx_copy, w_copy, s_mask, s_idx, s_w);
    __syncthreads();
    for (int e = threadIdx.x; e < n_experts; e += kRouteThreads) {
        const int c = __popc(s_mask[e]);
        hist_step[e] = c;                                // the step's activation vector
        if (c) hits[e] += c;                             // this workgroup is the step's only writer of H
    }
    dispatch_small(da, s_mask, s_slot_of, s_eis, s_idx, s_w, s_work);
}
#undef EXPERT_OF

__global__ void clear_i32_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// 256 threads, 1024 pairs per block, counted in LDS first (see topk_gate_kernel).
__global__ __launch_bounds__(256) void count_pairs_kernel(const int32_t* __restrict__ topk_idx, int n_pairs, int n_experts,
                                                          int32_t* hist_step) {
    __shared__ int32_t s_hist[kMaxExperts];
    for (int e = threadIdx.x; e < n_experts; e += 256) s_hist[e] = 0;
    __syncthreads();
    for (int q = 0; q < 4; ++q) {
        const int p = blockIdx.x * 1024 + q * 256 + threadIdx.x;
        if (p < n_pairs) {
            const int e = topk_idx[p];
            if (e >= 0 && e < n_experts) atomicAdd(&s_hist[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < n_experts; e += 256) {
        const int c = s_hist[e];
        if (c) atomicAdd(&hist_step[e], c);           // H += hist_step follows in the split kernel (one writer)
    }
}

}  // namespace

constexpr int kWideMinTokens = 256;       // steps of at least this many tokens take the 64-expert x 128-token kernel

int router_k_splits(const Shape& s, int n_tokens) {
    const int chunks = s.d / 32;
    int ks = 1;
    if (n_tokens >= kWideMinTokens) {
        // enough workgroups for every compute unit; a slice is a whole number of 128-column stages
        const int base = ((s.E + 63) / 64) * ((n_tokens + kWideTokens - 1) / kWideTokens);
        while (ks < kMaxRouterSplits && base * ks < 256 && chunks % (ks * 2 * kWideStageChunks) == 0) ks *= 2;
        return ks;
    }
    // enough workgroups to spread the router matrix over the chip when the token count is small
    const int base = ((s.E + 15) / 16) * ((n_tokens + 31) / 32);
    while (ks < kMaxRouterSplits && base * ks < 64 && chunks % (ks * 2) == 0 && chunks / (ks * 2) >= kRouterWaves) ks *= 2;
    return ks;
}

hipError_t launch_router_logits(const Shape& s, const uint16_t* x, int n_tokens, const float* w_r, float* z_part,
                                int32_t* hist_step_to_clear, hipStream_t stream, LaunchEvents ev) {
    const int ks = router_k_splits(s, n_tokens);
    const int e_pad = (s.E + 15) / 16 * 16;
    if (n_tokens >= kWideMinTokens && (s.d / 32) % (ks * kWideStageChunks) == 0) {
        dim3 grid(((s.E + 63) / 64) * ks, (n_tokens + kWideTokens - 1) / kWideTokens);
        TIDE_LAUNCH(router_logits_wide_kernel, grid, dim3(kRouterWaves * 64), stream, ev, x, n_tokens, s.d, s.E,
                    e_pad, ks, w_r, z_part, hist_step_to_clear);
    } else if (n_tokens >= kWideMinTokens) {
        dim3 grid(((s.E + 15) / 16) * ks, (n_tokens + 63) / 64);
        TIDE_LAUNCH(router_logits_kernel<4>, grid, dim3(kRouterWaves * 64), stream, ev, x, n_tokens, s.d, s.E,
                           e_pad, ks, w_r, z_part, hist_step_to_clear);
    } else {
        dim3 grid(((s.E + 15) / 16) * ks, (n_tokens + 31) / 32);
        TIDE_LAUNCH(router_logits_kernel<2>, grid, dim3(kRouterWaves * 64), stream, ev, x, n_tokens, s.d, s.E,
                           e_pad, ks, w_r, z_part, hist_step_to_clear);
    }
    return hipGetLastError();
}

hipError_t launch_topk_gate(const Shape& s, const float* z_part, const float* bias, int n_tokens,
                            int32_t* topk_idx, float* topk_w, int32_t* hist_step,
                            int32_t* idx_copy, float* w_copy, hipStream_t stream, LaunchEvents ev) {
    const int ks = router_k_splits(s, n_tokens);
    const int e_pad = (s.E + 15) / 16 * 16;
    dim3 grid((n_tokens + 15) / 16);
    if (s.E <= 256) {
        TIDE_LAUNCH(topk_gate_kernel<16>, grid, dim3(256), stream, ev, z_part, ks, e_pad, bias, n_tokens, s.E, s.k,
                           s.gating, s.bias_mode, topk_idx, topk_w, hist_step, idx_copy, w_copy);
    } else {
        TIDE_LAUNCH(topk_gate_kernel<32>, grid, dim3(256), stream, ev, z_part, ks, e_pad, bias, n_tokens, s.E, s.k,
                           s.gating, s.bias_mode, topk_idx, topk_w, hist_step, idx_copy, w_copy);
    }
    return hipGetLastError();
}

bool routes_in_one_workgroup(const Shape& s, int n_tokens) {
    return n_tokens <= kSmallDispatchMaxTokens && n_tokens * s.k <= kSmallDispatchMaxPairs;
}

hipError_t launch_route_small(const Shape& s, const LayerTables& t, const Workspace& w, const float* bias, int n_tokens,
                              int32_t* idx_copy, float* w_copy, tide_miss* miss, int miss_cap, int32_t* n_miss,
                              hipStream_t stream, LaunchEvents ev) {
    const int ks = router_k_splits(s, n_tokens);
    const int e_pad = (s.E + 15) / 16 * 16;
    DispatchArgs da;
    da.n_tokens = n_tokens; da.k = s.k; da.capacity = s.capacity; da.n_shared = s.n_shared; da.n_experts = s.E;
    da.slot_of = t.slot_of; da.expert_in_slot = t.expert_in_slot; da.expert_p12 = t.expert_p12; da.row_token = w.row_token; da.pair_row = w.pair_row;
    da.slot_off = w.slot_off; da.tasks = w.tasks; da.n_tasks = w.n_tasks; da.miss = miss; da.miss_cap = miss_cap;
    da.n_miss = n_miss; da.counters = w.counters;
    if (s.E <= 256)
        TIDE_LAUNCH(route_small_kernel<16>, dim3(1), dim3(kRouteThreads), stream, ev, w.logits, ks, e_pad, bias, s.E, s.gating,
                    s.bias_mode, w.topk_idx, w.topk_w, w.hist_step, t.hits, idx_copy, w_copy, da);
    else
        TIDE_LAUNCH(route_small_kernel<32>, dim3(1), dim3(kRouteThreads), stream, ev, w.logits, ks, e_pad, bias, s.E, s.gating,
                    s.bias_mode, w.topk_idx, w.topk_w, w.hist_step, t.hits, idx_copy, w_copy, da);
    return hipGetLastError();
}

hipError_t launch_clear_i32(int32_t* p, int n, hipStream_t stream) {
    hipLaunchKernelGGL(clear_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
    return hipGetLastError();
}

hipError_t launch_count_pairs(const Shape& s, const int32_t* topk_idx, int n_tokens, int32_t* hist_step,
                              hipStream_t stream) {
    hipLaunchKernelGGL(clear_i32_kernel, dim3((s.E + 255) / 256), dim3(256), 0, stream, hist_step, s.E);
    const int n_pairs = n_tokens * s.k;
    hipLaunchKernelGGL(count_pairs_kernel, dim3((n_pairs + 1023) / 1024), dim3(256), 0, stream, topk_idx, n_pairs,
                       s.E, hist_step);
    return hipGetLastError();
}

}  // namespace tide
