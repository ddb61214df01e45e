// Grouped SwiGLU expert GEMMs over the resident experts that have tokens this step
// (Alg. 1: "output = e(x)" for tokens whose expert is in E^GPU; Eq. 1-2: Lat^GPU).
//
//   pass 0:  act[row][:]  = silu(Wg x_row) * (Wu x_row)      bf16 out, fp32 accumulate
//   pass 1:  y[row][:]    = Wd act[row][:]                   fp32 out
//
// At a diffusion block's size most experts see only a handful of tokens, so each
// weight element is used once per step: the kernels are weight streamers.  Weights
// are stored pre-tiled in the order a wavefront consumes them (tide_pack_expert): one
// 16-row x 32-column bf16 tile is 1 KiB, lane l's 16 bytes are the A operand of
// v_mfma_f32_16x16x32_bf16 for row l%16, columns (l/16)*8..+7.  A wave therefore
// fetches each tile with one fully coalesced 1 KiB load straight into registers --
// no LDS staging for weights.  Tokens sit on the MFMA's 16-wide N side.
#include "tide_internal.h"

namespace tide {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWaves = 4;            // independent waves per workgroup, each streaming its own weight rows
constexpr int kTileElems = 16 * 32;  // one packed tile

__device__ inline uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ inline float silu(float g) { return g / (1.f + __expf(-g)); }

constexpr int kPhaseCols = 512;                 // activation columns staged in LDS at a time
constexpr int kPhaseChunks = kPhaseCols / 32;
constexpr int kLdsRowElems = kPhaseCols + 8;    // +16 B per row: the 16 rows of a fragment read hit distinct banks

// grid.x = feature tile, grid.y = work item (blocks past *n_tasks leave at once).
// PASS 0 (RT = 2): wave w of feature tile ft owns SwiGLU columns (4*ft + w)*16 .. +15: one gate
//         tile and the matching up tile; K = d; activations gathered from hidden[row_token[row]].
// PASS 1 (RT = 4): wave w owns output columns (4*ft + w)*64 .. +63: four down tiles; K = d_ff;
//         activations = act[row].
//
// Weights: every wave streams its own row tiles from HBM straight into a ring of registers
// that runs D chunks (D * RT KiB) ahead of the matrix cores -- what hides HBM latency when each
// weight byte is used once.  Activations: the work item's token rows are shared by the
// workgroup's waves, so they are staged through LDS, 512 columns at a time; the next stage's
// rows are already in flight while the current one is consumed.
template <int PASS, int NT, int D>
__device__ inline void gemm_task(const uint16_t* const (&wt)[PASS == 0 ? 2 : 4], bool active, const Task& task,
                                 const uint16_t* __restrict__ act_in, const int32_t* __restrict__ row_token, int K,
                                 int n_out, int col0, uint16_t* __restrict__ act_out, float* __restrict__ y_out,
                                 uint16_t* lds) {
    constexpr int RT = PASS == 0 ? 2 : 4;
    constexpr int kPieces = NT * 4;                  // 16-byte pieces each thread stages per phase
    const int lane = threadIdx.x & 63;
    const int kchunks = K >> 5;

    // staging map: piece q = tid + 256*j covers row q/64 of the item, columns (q%64)*8 .. +7 of the phase
    const uint16_t* xsrc[kPieces];
#pragma unroll
    for (int j = 0; j < kPieces; ++j) {
        const int q = threadIdx.x + 256 * j;
        int r = q >> 6;
        if (r >= task.nrows) r = 0;                  // padding rows mirror a valid row; never stored
        const int row = task.row0 + r;
        const int64_t src = (PASS == 0) ? (int64_t)row_token[row] : (int64_t)row;
        xsrc[j] = act_in + src * K + (q & 63) * 8;
    }
    uint4 xr[kPieces];
    auto fetch_phase = [&](int phase) {
        const int width = min(kPhaseCols, K - phase * kPhaseCols);
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int c8 = ((threadIdx.x + 256 * j) & 63) * 8;
            xr[j] = (c8 < width) ? *reinterpret_cast<const uint4*>(xsrc[j] + phase * kPhaseCols) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_phase = [&]() {
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int q = threadIdx.x + 256 * j;
            *reinterpret_cast<uint4*>(lds + (q >> 6) * kLdsRowElems + (q & 63) * 8) = xr[j];
        }
    };
    fetch_phase(0);

    bf16x8 a[D][RT];
    if (active) {
#pragma unroll
        for (int i = 0; i < D; ++i)
            if (i < kchunks) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    a[i][r] = *reinterpret_cast<const bf16x8*>(wt[r] + (int64_t)i * kTileElems + lane * 8);
            }
    }
    f32x4 acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this lane's fragment position inside a staged row block
    const uint16_t* frag = lds + (lane & 15) * kLdsRowElems + (lane >> 4) * 8;

    for (int base = 0; base < kchunks; base += D) {
        if ((base & (kPhaseChunks - 1)) == 0) {
            const int phase = base / kPhaseChunks;
            if (phase) __syncthreads();              // everyone is done reading the previous stage
            store_phase();
            __syncthreads();
            if ((phase + 1) * kPhaseChunks < kchunks) fetch_phase(phase + 1);
        }
        if (active) {
#pragma unroll
            for (int i = 0; i < D; ++i) {
                const int c = base + i;
                if (c < kchunks) {
                    bf16x8 b[NT];
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        b[t] = *reinterpret_cast<const bf16x8*>(frag + t * 16 * kLdsRowElems + (c & (kPhaseChunks - 1)) * 32);
#pragma unroll
                    for (int r = 0; r < RT; ++r)
#pragma unroll
                        for (int t = 0; t < NT; ++t)
                            acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i][r], b[t], acc[r][t], 0, 0, 0);
                    const int cn = c + D;
                    if (cn < kchunks) {
#pragma unroll
                        for (int r = 0; r < RT; ++r)
                            a[i][r] = *reinterpret_cast<const bf16x8*>(wt[r] + (int64_t)cn * kTileElems + lane * 8);
                    }
                }
            }
        }
    }
    if (!active) return;

    // MFMA result layout: lane holds token column lane%16, feature rows (lane/16)*4 .. +3 of each tile.
    const int f4 = (lane >> 4) * 4;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int rr = t * 16 + (lane & 15);
        if (rr >= task.nrows) continue;
        const int64_t row = task.row0 + rr;
        if (PASS == 0) {
            const f32x4 g = acc[0][t], u = acc[1][t];
            const uint32_t a0 = f32_to_bf16_rne(silu(g[0]) * u[0]);
            const uint32_t a1 = f32_to_bf16_rne(silu(g[1]) * u[1]);
            const uint32_t a2 = f32_to_bf16_rne(silu(g[2]) * u[2]);
            const uint32_t a3 = f32_to_bf16_rne(silu(g[3]) * u[3]);
            uint2 pk;
            pk.x = a0 | (a1 << 16);
            pk.y = a2 | (a3 << 16);
            *reinterpret_cast<uint2*>(act_out + row * n_out + col0 + f4) = pk;
        } else {
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const f32x4 v = acc[r][t];
                *reinterpret_cast<float4*>(y_out + row * n_out + col0 + r * 16 + f4) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

template <int PASS>
__global__ __launch_bounds__(kWaves * 64) void expert_gemm_kernel(
    const uint16_t* __restrict__ slots, int64_t blob_elems, int64_t off_a, int64_t off_b,
    const Task* __restrict__ tasks, const int32_t* __restrict__ n_tasks, const uint16_t* __restrict__ act_in,
    const int32_t* __restrict__ row_token, int K, int n_out, uint16_t* __restrict__ act_out,
    float* __restrict__ y_out) {
    constexpr int RT = PASS == 0 ? 2 : 4;
    __shared__ __attribute__((aligned(16))) uint16_t lds[kRowsPerTask * kLdsRowElems];
    const int task_id = blockIdx.y;
    if (task_id >= *n_tasks) return;
    const int wave = threadIdx.x >> 6;
    const int wtile = blockIdx.x * kWaves + wave;            // this wave's group of RT row tiles
    const int col0 = wtile * (PASS == 0 ? 16 : 64);          // first output column of the wave
    const bool active = col0 < n_out;                        // spare waves still help staging
    const Task task = tasks[task_id];
    const int kchunks = K >> 5;
    const uint16_t* blob = slots + (int64_t)task.slot * blob_elems;
    const int64_t tile_stride = (int64_t)kchunks * kTileElems;   // one 16-row tile across all of K

    const uint16_t* wt[RT];
    if (PASS == 0) {
        wt[0] = blob + off_a + (int64_t)wtile * tile_stride;
        wt[1] = blob + off_b + (int64_t)wtile * tile_stride;
    } else {
#pragma unroll
        for (int r = 0; r < RT; ++r) wt[r] = blob + off_a + (int64_t)(wtile * 4 + r) * tile_stride;
    }
    const int nt = (task.nrows + 15) >> 4;
    static_assert(kRowsPerTask == 32, "one or two 16-token tiles per work item");
    if (nt == 1)
        gemm_task<PASS, 1, (PASS == 0 ? 8 : 4)>(wt, active, task, act_in, row_token, K, n_out, col0, act_out, y_out, lds);
    else
        gemm_task<PASS, 2, (PASS == 0 ? 8 : 4)>(wt, active, task, act_in, row_token, K, n_out, col0, act_out, y_out, lds);
}

}  // namespace

hipError_t launch_expert_gemm(int pass, const Shape& s, const LayerTables& t, const Workspace& w, const uint16_t* x,
                              int n_tokens, int max_tasks, hipStream_t stream, LaunchEvents ev) {
    (void)n_tokens;
    dim3 block(kWaves * 64);
    if (pass == 0) {
        TIDE_LAUNCH(expert_gemm_kernel<0>, dim3((s.I + 63) / 64, max_tasks), block, stream, ev, t.slots, s.blob_elems,
                           blob_off_gate(s), blob_off_up(s), w.tasks, w.n_tasks, x, w.row_token, s.d, s.I, w.act,
                           (float*)nullptr);
    } else {
        TIDE_LAUNCH(expert_gemm_kernel<1>, dim3((s.d + 255) / 256, max_tasks), block, stream, ev, t.slots, s.blob_elems,
                           blob_off_down(s), (int64_t)0, w.tasks, w.n_tasks, w.act, w.row_token, s.I, s.d,
                           (uint16_t*)nullptr, w.y);
    }
    return hipGetLastError();
}

}  // namespace tide
