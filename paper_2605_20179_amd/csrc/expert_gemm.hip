// Grouped SwiGLU expert GEMMs over the resident experts that have tokens this step
// (Alg. 1: "output = e(x)" for tokens whose expert is in E^GPU; Eq. 1-2: Lat^GPU).
//
//   pass 0:  act[row][:]  = silu(Wg x_row) * (Wu x_row)      bf16 out, fp32 accumulate
//   pass 1:  y[row][:]    = Wd act[row][:]                   fp32 out
//
// At a diffusion block's size most experts see only a handful of tokens, so each
// weight element is used once per step: the kernels are weight streamers.  Weights
// are stored pre-tiled in the order a wavefront consumes them (see pack.cpp): one
// 16-row x 32-column bf16 tile is 1 KiB, lane l's 16 bytes are the A operand of
// v_mfma_f32_16x16x32_bf16 for row l%16, columns (l/16)*8..+7.  A wave therefore
// fetches each tile with one fully coalesced 1 KiB load straight into registers --
// no LDS staging for weights.  Tokens sit on the MFMA's 16-wide N side.
#include "tide_internal.h"

namespace tide {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWaves = 4;            // waves per workgroup; they split the contraction (K) dimension
constexpr int kRowTiles = 4;         // 16-row weight tiles per workgroup
constexpr int kTokTiles = kRowsPerTask / 16;
constexpr int kTileElems = 16 * 32;  // one packed tile

__device__ inline uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ inline float silu(float g) { return g / (1.f + __expf(-g)); }

template <int NT>
__device__ inline void stream_k(const uint16_t* const (&wt)[kRowTiles], const uint16_t* const (&arow)[kTokTiles],
                                int wave, int lane, int kchunks, f32x4 (&acc)[kRowTiles][kTokTiles]) {
#pragma unroll 2
    for (int kc = wave; kc < kchunks; kc += kWaves) {
        bf16x8 a[kRowTiles], b[NT];
#pragma unroll
        for (int r = 0; r < kRowTiles; ++r)
            a[r] = *reinterpret_cast<const bf16x8*>(wt[r] + (int64_t)kc * kTileElems + lane * 8);
#pragma unroll
        for (int t = 0; t < NT; ++t) b[t] = *reinterpret_cast<const bf16x8*>(arow[t] + kc * 32);
#pragma unroll
        for (int r = 0; r < kRowTiles; ++r)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[r], b[t], acc[r][t], 0, 0, 0);
    }
}

// grid.x = feature tile, grid.y = work item (blocks past *n_tasks leave at once).
// PASS 0: feature tile = 32 SwiGLU columns (2 gate tiles + the matching 2 up tiles), K = d,
//         activations gathered from hidden[row_token[row]].
// PASS 1: feature tile = 64 output columns (4 down tiles), K = d_ff, activations = act[row].
template <int PASS>
__global__ __launch_bounds__(kWaves * 64) void expert_gemm_kernel(
    const uint16_t* __restrict__ slots, int64_t blob_elems, int64_t off_a, int64_t off_b,
    const Task* __restrict__ tasks, const int32_t* __restrict__ n_tasks, const uint16_t* __restrict__ act_in,
    const int32_t* __restrict__ row_token, int K, int out_ld, uint16_t* __restrict__ act_out,
    float* __restrict__ y_out) {
    const int task_id = blockIdx.y;
    if (task_id >= *n_tasks) return;
    const Task task = tasks[task_id];
    const int ft = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int kchunks = K >> 5;
    const uint16_t* blob = slots + (int64_t)task.slot * blob_elems;
    const int64_t tile_stride = (int64_t)kchunks * kTileElems;   // one 16-row tile across all of K

    const uint16_t* wt[kRowTiles];
    if (PASS == 0) {
        wt[0] = blob + off_a + (int64_t)(2 * ft) * tile_stride;
        wt[1] = blob + off_a + (int64_t)(2 * ft + 1) * tile_stride;
        wt[2] = blob + off_b + (int64_t)(2 * ft) * tile_stride;
        wt[3] = blob + off_b + (int64_t)(2 * ft + 1) * tile_stride;
    } else {
#pragma unroll
        for (int r = 0; r < kRowTiles; ++r) wt[r] = blob + off_a + (int64_t)(4 * ft + r) * tile_stride;
    }

    const uint16_t* arow[kTokTiles];
#pragma unroll
    for (int t = 0; t < kTokTiles; ++t) {
        int r = t * 16 + (lane & 15);
        if (r >= task.nrows) r = 0;                       // padding lanes read a valid row; never stored
        const int row = task.row0 + r;
        const int64_t src = (PASS == 0) ? (int64_t)row_token[row] : (int64_t)row;
        arow[t] = act_in + src * K + (lane >> 4) * 8;
    }

    f32x4 acc[kRowTiles][kTokTiles];
#pragma unroll
    for (int r = 0; r < kRowTiles; ++r)
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nt = (task.nrows + 15) >> 4;
    switch (nt) {
        case 1: stream_k<1>(wt, arow, wave, lane, kchunks, acc); break;
        case 2: stream_k<2>(wt, arow, wave, lane, kchunks, acc); break;
        case 3: stream_k<3>(wt, arow, wave, lane, kchunks, acc); break;
        default: stream_k<4>(wt, arow, wave, lane, kchunks, acc); break;
    }

    // Sum the waves' K-partials through LDS in a fixed order; wave w ends up owning token tile w.
    __shared__ f32x4 red[kWaves][kTokTiles][64];
    f32x4 res[kRowTiles];
#pragma unroll
    for (int r = 0; r < kRowTiles; ++r) {
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) red[wave][t][lane] = acc[r][t];
        __syncthreads();
        res[r] = red[0][wave][lane] + red[1][wave][lane] + red[2][wave][lane] + red[3][wave][lane];
        __syncthreads();
    }

    // MFMA result layout: lane holds token column lane%16, feature rows (lane/16)*4 .. +3 of each tile.
    const int rr = wave * 16 + (lane & 15);
    if (rr >= task.nrows) return;
    const int64_t row = task.row0 + rr;
    const int f4 = (lane >> 4) * 4;
    if (PASS == 0) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const f32x4 g = res[r], u = res[r + 2];
            const uint32_t a0 = f32_to_bf16_rne(silu(g[0]) * u[0]);
            const uint32_t a1 = f32_to_bf16_rne(silu(g[1]) * u[1]);
            const uint32_t a2 = f32_to_bf16_rne(silu(g[2]) * u[2]);
            const uint32_t a3 = f32_to_bf16_rne(silu(g[3]) * u[3]);
            uint2 pk;
            pk.x = a0 | (a1 << 16);
            pk.y = a2 | (a3 << 16);
            *reinterpret_cast<uint2*>(act_out + row * out_ld + ft * 32 + r * 16 + f4) = pk;
        }
    } else {
#pragma unroll
        for (int r = 0; r < kRowTiles; ++r) {
            const f32x4 v = res[r];
            *reinterpret_cast<float4*>(y_out + row * out_ld + ft * 64 + r * 16 + f4) =
                make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

}  // namespace

hipError_t launch_expert_gemms(const Shape& s, const LayerTables& t, const Workspace& w, const uint16_t* x,
                               int n_tokens, int max_tasks, hipStream_t stream) {
    (void)n_tokens;
    dim3 block(kWaves * 64);
    hipLaunchKernelGGL(expert_gemm_kernel<0>, dim3(s.I / 32, max_tasks), block, 0, stream, t.slots, s.blob_elems,
                       blob_off_gate(s), blob_off_up(s), w.tasks, w.n_tasks, x, w.row_token, s.d, s.I, w.act,
                       (float*)nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(expert_gemm_kernel<1>, dim3(s.d / 64, max_tasks), block, 0, stream, t.slots, s.blob_elems,
                       blob_off_down(s), (int64_t)0, w.tasks, w.n_tasks, w.act, w.row_token, s.I, s.d,
                       (uint16_t*)nullptr, w.y);
    return hipGetLastError();
}

}  // namespace tide
