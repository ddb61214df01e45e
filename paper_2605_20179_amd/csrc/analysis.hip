// Refresh-interval analysis on per-step expert activation counts counts[t][e] (int32):
// routing stability across denoising steps (Sec. 3.2: cosine similarity of the steps' activation
// vectors, Fig. 1a / Fig. 2b; distinct experts per step, Fig. 2a), the drift rate of the optimal
// placement (Eq. 4), and the cost model that picks the interval (Eq. 5-7).
#include "tide_internal.h"

#include <cmath>

namespace tide {

namespace {

constexpr int kAnaThreads = 256;

__device__ inline long long block_sum_ll(long long v, long long* lds) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();                                     // lds may still be read from the last call
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    long long t = 0;
#pragma unroll
    for (int w = 0; w < kAnaThreads / 64; ++w) t += lds[w];
    return t;
}

// grid (n_steps, n_steps): block (j, i) writes sim[i][j]; the dot products of small integers are exact
// in 64-bit integers, the quotient is formed once in fp64.  Blocks of column 0 also count the distinct
// experts of their step.
__global__ __launch_bounds__(kAnaThreads) void similarity_kernel(const int32_t* __restrict__ counts, int n_experts,
                                                                 double* __restrict__ sim, int32_t* __restrict__ unique) {
    __shared__ long long lds[kAnaThreads / 64];
    const int j = blockIdx.x, i = blockIdx.y, n_steps = gridDim.x;
    const int32_t* ci = counts + (int64_t)i * n_experts;
    const int32_t* cj = counts + (int64_t)j * n_experts;
    long long dot = 0, ni = 0, nj = 0, nz = 0;
    for (int e = threadIdx.x; e < n_experts; e += kAnaThreads) {
        const long long a = ci[e], b = cj[e];
        dot += a * b;
        ni += a * a;
        nj += b * b;
        nz += a > 0 ? 1 : 0;
    }
    dot = block_sum_ll(dot, lds);
    ni = block_sum_ll(ni, lds);
    nj = block_sum_ll(nj, lds);
    nz = block_sum_ll(nz, lds);
    if (threadIdx.x == 0) {
        if (sim) sim[(int64_t)i * n_steps + j] = (ni > 0 && nj > 0) ? (double)dot / (sqrt((double)ni) * sqrt((double)nj)) : 0.0;
        if (unique && j == 0) unique[i] = (int)nz;
    }
}

// block t: the top-`budget` sets of steps t and t-1 under (count descending, lower expert first) by
// all-pairs ranks; drift[t] = |set_t \ set_{t-1}| / budget (Eq. 4), drift[0] = 0.
__global__ __launch_bounds__(kAnaThreads) void drift_kernel(const int32_t* __restrict__ counts, int n_experts, int budget,
                                                            double* __restrict__ drift) {
    __shared__ long long lds[kAnaThreads / 64];
    __shared__ int32_t cur[kMaxExperts], prev[kMaxExperts];
    const int t = blockIdx.x;
    if (t == 0) {
        if (threadIdx.x == 0) drift[0] = 0.0;
        return;
    }
    for (int e = threadIdx.x; e < n_experts; e += kAnaThreads) {
        cur[e] = counts[(int64_t)t * n_experts + e];
        prev[e] = counts[(int64_t)(t - 1) * n_experts + e];
    }
    __syncthreads();
    long long entered = 0;
    for (int e = threadIdx.x; e < n_experts; e += kAnaThreads) {
        int rank_cur = 0, rank_prev = 0;
        const int ce = cur[e], pe = prev[e];
        for (int q = 0; q < n_experts; ++q) {
            rank_cur += (cur[q] > ce || (cur[q] == ce && q < e)) ? 1 : 0;
            rank_prev += (prev[q] > pe || (prev[q] == pe && q < e)) ? 1 : 0;
        }
        entered += (rank_cur < budget && rank_prev >= budget) ? 1 : 0;
    }
    entered = block_sum_ll(entered, lds);
    if (threadIdx.x == 0) drift[t] = (double)entered / (double)budget;
}

}  // namespace

hipError_t launch_routing_stability(const int32_t* counts, int n_steps, int n_experts, int budget, double* sim,
                                    int32_t* unique, double* drift, hipStream_t stream) {
    if (sim || unique) {
        hipLaunchKernelGGL(similarity_kernel, dim3(sim ? n_steps : 1, n_steps), dim3(kAnaThreads), 0, stream, counts,
                           n_experts, sim, unique);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (drift) hipLaunchKernelGGL(drift_kernel, dim3(n_steps), dim3(kAnaThreads), 0, stream, counts, n_experts, budget, drift);
    return hipGetLastError();
}

// Eq. 5 and Eq. 6 for tau = 1 .. n_steps-1 (host, fp64):
//   lat_io[tau-1]  = c_io * (B*T/tau) * (1 - (1-d)^tau)        lat_cpu[tau-1] = c_cpu * T * B * f[tau-1]
void interval_costs(int budget, int n_steps, double d, double c_io, double c_cpu, const double* f, double* lat_io,
                    double* lat_cpu) {
    for (int tau = 1; tau < n_steps; ++tau) {
        lat_io[tau - 1] = c_io * ((double)((int64_t)budget * n_steps) / (double)tau * (1.0 - std::pow(1.0 - d, (double)tau)));
        lat_cpu[tau - 1] = c_cpu * (double)n_steps * (double)budget * f[tau - 1];
    }
}

}  // namespace tide
