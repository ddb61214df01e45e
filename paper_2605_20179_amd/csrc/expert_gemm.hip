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
// no LDS staging for weights.  The tiles of the stripes a workgroup consumes together
// are stored K chunk by K chunk, so the workgroup reads one contiguous region front to
// back (all memory channels in turn) instead of 16 streams 128 KiB apart.  Tokens sit
// on the MFMA's 16-wide N side.
#include "packed12_device.h"
#include "tide_internal.h"

#include <type_traits>

namespace tide {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWaves = 4;            // independent waves per workgroup, each streaming its own weight rows
constexpr int kTileElems = 16 * 32;  // one packed tile

// The two forms a cache slot can hold its blob in.  bf16: tiles of 1 KiB, a lane's 16 bytes are its MFMA operand as they
// are.  12-bit (packed12.h): tile payloads of 768 bytes, 12 per lane, plus a 16-byte table per tile; the wave decodes
// its operand in registers, so 3/4 of the bytes leave HBM for the same weights.
constexpr int kFmtBf16 = 0, kFmtP12 = 1;
template <int FMT>
struct WeightFormat;
template <>
struct WeightFormat<kFmtBf16> {
    typedef bf16x8 Word;                                      // what a lane keeps in the ring per tile
    static constexpr int kTileStride = kTileElems;            // uint16 units from one tile to the next
    static constexpr int kLaneStride = 8;                     // uint16 units from one lane's piece to the next
    static constexpr int kPayloadOff = 0;                     // uint16 units from the blob's start to tile 0
};
template <>
struct WeightFormat<kFmtP12> {
    typedef P12Words Word;
    static constexpr int kTileStride = kP12TileBytes / 2;
    static constexpr int kLaneStride = 6;
    static constexpr int kPayloadOff = kP12HeaderBytes / 2;
};

__device__ inline uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// A weight tile is normally used once by the wave that fetches it: a non-temporal load keeps it from taking a
// line of the vector cache (a plain streaming kernel reads 6.5 TB/s this way against 5.8 TB/s with ordinary loads).
// When a slot is cut into several small items (SHARED), their workgroups read the same tiles at about the same
// time: ordinary loads let the later readers find them in L2.
template <bool SHARED>
__device__ inline void load_weights(const uint16_t* p, bf16x8& w) {
    if (SHARED) w = *reinterpret_cast<const bf16x8*>(p);
    else w = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p));
}
template <bool SHARED>
__device__ inline void load_weights(const uint16_t* p, P12Words& w) {       // 12 bytes, dword-aligned
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    if (SHARED) {
        w.a0 = q[0];
        w.a1 = q[1];
        w.b = q[2];
    } else {
        w.a0 = __builtin_nontemporal_load(q);
        w.a1 = __builtin_nontemporal_load(q + 1);
        w.b = __builtin_nontemporal_load(q + 2);
    }
}
__device__ inline bf16x8 mfma_operand(const bf16x8& w, const uint4&) { return w; }
__device__ inline bf16x8 mfma_operand(const P12Words& w, const uint4& table) {
    return __builtin_bit_cast(bf16x8, p12_decode(w, table));
}

__device__ inline float silu(float g) { return g / (1.f + __expf(-g)); }

// Shared skeleton of the small (<= 32 rows) and large (<= 256 rows) work-item kernels.
//
//   PASS 0: a wave owns G gate stripes and the G matching up stripes (RT = 2G weight stripes of
//           16 rows), i.e. SwiGLU columns wtile*16G .. +16G-1; K = d; activations are gathered
//           from hidden[row_token[row]].
//   PASS 1: a wave owns RT consecutive down stripes, i.e. output columns wtile*16RT .. ; K = d_ff;
//           activations = act[row].
//
// Weights: every wave streams its own stripes from HBM (or L2, when several work items share a
// slot) straight into a ring of registers that runs D chunks ahead of the matrix cores -- what
// hides memory latency when each weight byte is used once.  Activations: the work item's token
// rows are shared by the workgroup's four waves, so they are staged through LDS, PC chunks of 32
// columns at a time; the next stage's rows are already in flight while the current one is used.
// Tokens sit on the MFMA's 16-wide N side, NT token tiles per work item.
// Where a wave finds its weight stripes: a wave's stripes all lie in one group of the packed layout, and inside a
// group the K chunk is the slow index, so chunk c of stripe r is tile  first + stripe_tile(r) + c * cstep  of the blob.
// Everything here is the same for all lanes of a wave: it lives in scalar registers.
struct WeightStream {
    int first;                // tile index of the wave's first stripe (PASS 0: its first gate stripe), chunk 0
    int cstep;                // tiles from one K chunk to the next
    int up;                   // PASS 0: tiles from a gate stripe to the matching up stripe
    int table_first;          // 12-bit form: table slot of that first stripe, chunk 0 (tables are stored stripe first:
                              // stripe r, chunk c of the wave at table_first + stripe_tile(r) * chunks + c)
};

template <int PASS, int RT>
__device__ inline int stripe_tile(const WeightStream& ws, int r) {
    constexpr int G = RT / 2;
    if (PASS == 0 && r >= G) return ws.up + (r - G);
    return r;
}

// wtile: the wave's tile of output features (wave-uniform).  A spare wave (columns past n_out) streams the last valid
// wave's stripes and stores nothing: it stays in step with the barriers without a predicate around the loop.
// tile0: the blob's first tile of this pass (gate/up: 0, down: after the gate and up matrices).
template <int PASS, int RT>
__device__ inline void weight_stream(int tile0, int wtile, bool active, int K, int n_out, WeightStream& ws) {
    constexpr int G = RT / 2;                        // PASS 0: gate stripes per wave
    const int kchunks = K >> 5;
    const int wsrc = active ? wtile : (n_out / (16 * (PASS == 0 ? G : RT)) - 1);
    if (PASS == 0) {
        static_assert(PASS != 0 || kGateUpGroup % (RT / 2) == 0, "a wave's column blocks share a group");
        const int first = wsrc * G;                                  // the wave's first SwiGLU column block
        const int g = first / kGateUpGroup, j0 = first % kGateUpGroup;
        const int ng = min(kGateUpGroup, n_out / 16 - g * kGateUpGroup);
        ws.first = tile0 + g * 2 * kGateUpGroup * kchunks + j0;
        ws.cstep = 2 * ng;
        ws.up = ng;
        ws.table_first = tile0 + g * 2 * kGateUpGroup * kchunks + j0 * kchunks;
    } else {
        static_assert(PASS == 0 || kDownGroup % RT == 0, "a wave's stripes share a group");
        const int first = wsrc * RT;
        const int g = first / kDownGroup, j0 = first % kDownGroup;
        const int ng = min(kDownGroup, n_out / 16 - g * kDownGroup);
        ws.first = tile0 + g * kDownGroup * kchunks + j0;
        ws.cstep = ng;
        ws.up = 0;
        ws.table_first = tile0 + g * kDownGroup * kchunks + j0 * kchunks;
    }
}

template <int PASS, int RT, int NT, int D, int PC, int NBUF, bool SHARED = false, int FMT = kFmtBf16>
__device__ inline void gemm_task(const uint16_t* blob, int64_t off_w, int wtile, bool active,
                                 const Task& task, const uint16_t* __restrict__ act_in,
                                 const int32_t* __restrict__ row_token, int K, int n_out, int64_t blob_elems,
                                 uint16_t* __restrict__ act_out, float* __restrict__ y_out, uint16_t* lds, uint4* wave_tables) {
    static_assert(PC % D == 0 || (NBUF == 2 && D % PC == 0), "stage boundaries must fall on whole chunks of a ring turn");
    constexpr int G = RT / 2;                        // PASS 0: gate stripes per wave
    constexpr int kCols = PC * 32;                   // columns per stage
    constexpr int kRowElems = kCols + 8;             // +16 B per LDS row: a fragment's 16 rows hit distinct banks
    constexpr int kPPR = PC * 4;                     // 16-byte pieces per staged row
    constexpr int kPieces = NT * 16 * kPPR / 256;    // pieces each thread stages
    static_assert(NT * 16 * kPPR % 256 == 0, "staging must divide evenly over the workgroup");
    constexpr int kBufElems = NT * 16 * kRowElems;   // one staging buffer
    const int lane = threadIdx.x & 63;
    const int kchunks = K >> 5;
    const int col0 = wtile * 16 * (PASS == 0 ? G : RT);

    typedef WeightFormat<FMT> Fmt;
    WeightStream ws;
    weight_stream<PASS, RT>((int)(off_w / kTileElems), wtile, active, K, n_out, ws);
    const uint16_t* lane_base = blob + Fmt::kPayloadOff + lane * Fmt::kLaneStride;
    // chunk c of stripe r: scalar address arithmetic plus the lane's place in the tile
    auto tile = [&](int r, int c) {
        return lane_base + (int64_t)(ws.first + stripe_tile<PASS, RT>(ws, r) + c * ws.cstep) * Fmt::kTileStride;
    };

    // 12-bit form: the tables of the wave's next kTableChunks chunks (64 tiles: one per lane) come through a piece of
    // LDS that only this wave touches -- one 16-byte load per lane a block ahead, one store at the block's start, and
    // a broadcast read per tile when it is decoded.  A wave's LDS accesses complete in order: no barrier is needed.
    // Large items (kAhead) decode a chunk while the MFMAs of the chunk before it run: the decode of a block's first
    // chunk then falls into the block before, so their table blocks alternate between two buffers.
    constexpr bool kAhead = FMT == kFmtP12 && NBUF == 2;
    constexpr int kTableChunks = 64 / RT;
    static_assert(FMT == kFmtBf16 || (kTableChunks % D == 0 && D <= kTableChunks), "table blocks start on whole ring turns");
    const uint8_t* table0 = reinterpret_cast<const uint8_t*>(blob) + kP12HeaderBytes + (blob_elems / kTileElems) * kP12TileBytes;
    uint4 next_tables;
    auto fetch_tables = [&](int block) {
        const int c = min(block * kTableChunks + lane / RT, kchunks - 1), r = lane % RT;
        const int t = ws.table_first + ((PASS == 0 && r >= G) ? ws.up + (r - G) : r) * kchunks + c;
        next_tables = *reinterpret_cast<const uint4*>(table0 + (int64_t)t * kP12TableBytes);
    };
    auto table_block = [&](int block) {               // before the first decode of a block's chunks
        wave_tables[(kAhead ? (block & 1) * 64 : 0) + lane] = next_tables;
        fetch_tables(block + 1);
    };
    auto table_of = [&](int c, int r) {
        const unsigned cu = (unsigned)c;              // chunk indices are never negative: unsigned / and % are a shift and a mask
        return wave_tables[(kAhead ? ((cu / kTableChunks) & 1) * 64 : 0) + (cu % kTableChunks) * RT + r];
    };
    if (FMT == kFmtP12) fetch_tables(0);

    // staging map: piece q = tid + 256*j covers row q / kPPR of the item, columns (q % kPPR)*8 .. +7 of the
    // stage; kPPR divides 256, so a thread's pieces all sit at the same columns
    static_assert(256 % kPPR == 0, "a thread stages the same columns of each of its rows");
    const int xcol = (threadIdx.x % kPPR) * 8;
    const uint16_t* xsrc[kPieces];
#pragma unroll
    for (int j = 0; j < kPieces; ++j) {
        int r = (threadIdx.x + 256 * j) / kPPR;
        if (r >= task.nrows) r = 0;                  // padding rows mirror a valid row; never stored
        const int row = task.row0 + r;
        const int64_t src = (PASS == 0) ? (int64_t)row_token[row] : (int64_t)row;
        xsrc[j] = act_in + src * K;
    }
    u32x4 xr[kPieces];
    // columns past K (a last, partial stage) are clamped to the row's last piece: loaded, staged, never
    // read by an MFMA -- the loop body stays free of branches
    auto fetch_stage = [&](int stage) {
        const int col = min(stage * kCols + xcol, K - 8);
#pragma unroll
        for (int j = 0; j < kPieces; ++j) xr[j] = *reinterpret_cast<const u32x4*>(xsrc[j] + col);
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int q = threadIdx.x + 256 * j;
            *reinterpret_cast<u32x4*>(lds + buf * kBufElems + (q / kPPR) * kRowElems + (q % kPPR) * 8) = xr[j];
        }
    };
    const int last_stage = (kchunks - 1) / PC;
    fetch_stage(0);
    if (NBUF == 2) {
        // two buffers: stage s+1 is written while stage s is consumed, one barrier per stage
        store_stage(0);
        fetch_stage(min(1, last_stage));
    }

    // ring prologue (chunk indices past the end are clamped: a redundant in-bounds load, never used)
    typename Fmt::Word a[D][RT];
#pragma unroll
    for (int i = 0; i < D; ++i) {
        const int ci = min(i, kchunks - 1);
#pragma unroll
        for (int r = 0; r < RT; ++r) load_weights<SHARED>(tile(r, ci), a[i][r]);
    }
    f32x4 acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this lane's fragment position inside a staged 16-row block
    const uint16_t* frag = lds + (lane & 15) * kRowElems + (lane >> 4) * 8;
    // fragments of token tiles t0 .. t0+CNT-1 for chunk c
    auto read_frags = [&](bf16x8* b, int c, int t0, auto cnt) {
        const unsigned cu = (unsigned)c;
        const uint16_t* from = frag + (NBUF == 2 ? ((cu / PC) & 1) * kBufElems : 0) + (cu % PC) * 32;
#pragma unroll
        for (int t = 0; t < decltype(cnt)::value; ++t)
            b[t] = *reinterpret_cast<const bf16x8*>(from + (t0 + t) * 16 * kRowElems);
    };
    // chunk c (ring slot i) against token tiles t0 ..: a stripe's operand is the ring's word as it is, or is decoded
    // with the tile's table right before the stripe's MFMAs (the decode of the next stripe runs under them)
    auto mfmas = [&](const bf16x8* b, int c, int i, int t0, auto cnt) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            uint4 table{};
            if (FMT == kFmtP12) table = table_of(c, r);
            const bf16x8 w = mfma_operand(a[i][r], table);
#pragma unroll
            for (int t = 0; t < decltype(cnt)::value; ++t)
                acc[r][t0 + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, b[t], acc[r][t0 + t], 0, 0, 0);
        }
    };
    auto refill = [&](int c, int i) {
        const int cn = min(c + D, kchunks - 1);
#pragma unroll
        for (int r = 0; r < RT; ++r) load_weights<SHARED>(tile(r, cn), a[i][r]);
    };
    using all_tiles = std::integral_constant<int, NT>;

    if constexpr (NBUF == 1) {
        auto stage_switch = [&](int base) {
            const int stage = base / PC;
            if (stage) __syncthreads();              // everyone is done reading the previous stage
            store_stage(0);
            __syncthreads();
            if ((stage + 1) * PC < kchunks) fetch_stage(stage + 1);
        };
        // chunk c: MFMAs from ring slot i and the staged fragments, then refill the slot D chunks ahead
        auto chunk = [&](int c, int i) {
            bf16x8 b[NT];
            read_frags(b, c, 0, all_tiles{});
            mfmas(b, c, i, 0, all_tiles{});
            refill(c, i);
        };
        // the main loop is straight-line (no per-chunk predicates): whole turns of the ring
        int base = 0;
        for (; base + D <= kchunks; base += D) {
            if (FMT == kFmtP12 && base % kTableChunks == 0) table_block(base / kTableChunks);
            if (base % PC == 0) stage_switch(base);
#pragma unroll
            for (int i = 0; i < D; ++i) chunk(base + i, i);
        }
        if (base < kchunks) {                        // a last partial turn (K not a multiple of 32*D)
            if (FMT == kFmtP12 && base % kTableChunks == 0) table_block(base / kTableChunks);
            if (base % PC == 0) stage_switch(base);
#pragma unroll
            for (int i = 0; i < D; ++i)
                if (base + i < kchunks) chunk(base + i, i);
        }
    } else {
        // Fragments are double-buffered in registers too: the next set is read from LDS while the current
        // one feeds the MFMAs.  More than 8 token tiles are handled as two half sets per chunk, so the
        // fragment registers stay at 2 x 8 tiles.  The stage barrier sits right ahead of the read of the
        // next stage's first fragments, in the stage's last chunk: by then every thread has written its
        // part of the next stage (at the stage's first chunk) and every wave has read the stage before
        // this one to the end, so the buffer written at the next stage's first chunk is free.
        constexpr int NH = NT > 8 ? 2 : 1;           // half sets per chunk
        constexpr int NTH = NT / NH;
        static_assert(NT % NH == 0 && D % 2 == 0, "fragment buffers alternate with the step's parity");
        static_assert(PC % D == 0 || D % PC == 0, "stage boundaries must fall on whole chunks of a ring turn");
        using half_tiles = std::integral_constant<int, NTH>;
        bf16x8 b[2][NTH];
        // kAhead: the decoded operands of this chunk and of the next.  A chunk's tiles are decoded, a stripe or two per
        // half set, between the MFMAs of the chunk before it (a wave that keeps this many accumulators is alone on
        // its SIMD: whatever it issues beside an MFMA in flight is free, whatever it issues between two costs), and
        // the ring slot they came from is refilled at once.
        bf16x8 wdec[kAhead ? 2 : 1][RT];
        if constexpr (kAhead) {
            table_block(0);
#pragma unroll
            for (int r = 0; r < RT; ++r) wdec[0][r] = mfma_operand(a[0][r], table_of(0, r));
            refill(0, 0);
        }
        __syncthreads();                             // stage 0 is complete
        read_frags(b[0], 0, 0, half_tiles{});
        auto chunk = [&](int c, int i) {
            if ((unsigned)c % PC == 0) {
                // no branches in the loop body: past the last stage this stores a stage nobody reads into
                // the buffer that is free, and fetches the last stage once more
                const int stage = (unsigned)c / PC;
                store_stage((stage + 1) & 1);
                fetch_stage(min(stage + 2, last_stage));
            }
            // scheduling fences: the next fragments are requested before the current MFMAs start, and
            // each chunk's weight loads stay with its MFMAs, so the ring stays D chunks ahead
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const int q = NH == 2 ? h : (i & 1);     // parity of this step
                if (h == NH - 1) {
                    if ((unsigned)c % PC == PC - 1) __syncthreads();
                    read_frags(b[q ^ 1], min(c + 1, kchunks - 1), 0, half_tiles{});
                } else {
                    read_frags(b[q ^ 1], c, NTH, half_tiles{});
                }
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (kAhead) {
                    constexpr int RH = RT / NH;              // stripes of the next chunk decoded under this half set
                    static_assert(RT % NH == 0, "the next chunk's stripes divide over the half sets");
                    const int cn = min(c + 1, kchunks - 1), in = (i + 1) % D;
#pragma unroll
                    for (int r = 0; r < RT; ++r)
#pragma unroll
                        for (int t = 0; t < NTH; ++t)
                            acc[r][h * NTH + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wdec[i & 1][r], b[q][t], acc[r][h * NTH + t], 0, 0, 0);
#pragma unroll
                    for (int r = h * RH; r < (h + 1) * RH; ++r) wdec[(i + 1) & 1][r] = mfma_operand(a[in][r], table_of(cn, r));
                    if (h == NH - 1) refill(c + 1, in);
                    // the order asked of the scheduler: the table reads first, then every MFMA followed by its share
                    // of the decode's vector instructions
                    constexpr int kMfmas = RT * NTH, kPerMfma = (RH * 20 + kMfmas - 1) / kMfmas;
                    __builtin_amdgcn_sched_group_barrier(0x100, RH, 0);
#pragma unroll
                    for (int m = 0; m < kMfmas; ++m) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, kPerMfma, 0);
                    }
                } else {
                    mfmas(b[q], c, i, h * NTH, half_tiles{});
                    if (h == NH - 1) refill(c, i);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // a table block is put in place at the top of the ring turn in which its first chunk is decoded: the turn
        // that begins with it, or (kAhead) the turn before
        auto tables_for_turn = [&](int base) {
            const int first = kAhead ? base + D : base;
            if (FMT == kFmtP12 && first % kTableChunks == 0) table_block(first / kTableChunks);
        };
        int base = 0;
        for (; base + D <= kchunks; base += D) {
            tables_for_turn(base);
#pragma unroll
            for (int i = 0; i < D; ++i) chunk(base + i, i);
        }
        if (base < kchunks) {
            tables_for_turn(base);
#pragma unroll
            for (int i = 0; i < D; ++i)
                if (base + i < kchunks) chunk(base + i, i);
        }
    }
    if (!active) return;

    // MFMA result layout: lane holds token column lane%16, feature rows (lane/16)*4 .. +3 of each stripe.
    const int f4 = (lane >> 4) * 4;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int rr = t * 16 + (lane & 15);
        if (rr >= task.nrows) continue;
        const int64_t row = task.row0 + rr;
        if (PASS == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const f32x4 gt = acc[g][t], up = acc[g + G][t];
                const uint32_t a0 = f32_to_bf16_rne(silu(gt[0]) * up[0]);
                const uint32_t a1 = f32_to_bf16_rne(silu(gt[1]) * up[1]);
                const uint32_t a2 = f32_to_bf16_rne(silu(gt[2]) * up[2]);
                const uint32_t a3 = f32_to_bf16_rne(silu(gt[3]) * up[3]);
                uint2 pk;
                pk.x = a0 | (a1 << 16);
                pk.y = a2 | (a3 << 16);
                *reinterpret_cast<uint2*>(act_out + row * n_out + col0 + g * 16 + f4) = pk;
            }
        } else {
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const f32x4 v = acc[r][t];
                *reinterpret_cast<float4*>(y_out + row * n_out + col0 + r * 16 + f4) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

// Small work items: up to 32 rows of one slot (the whole slot at block 32 / batch 1).
// grid.x = feature tile, grid.y = work item (blocks past n_tasks[0] leave at once).
constexpr int kSmallPC = 16;       // 512 columns per stage
constexpr int kSmallRT0 = 2, kSmallD0 = 8;   // gate/up: weight stripes per wave, ring depth
constexpr int kSmallRT1 = 4, kSmallD1 = 4;   // down
// The same for a context whose slots keep the 12-bit form (P12SLOTS): a 12-bit tile is 3 registers in the ring
// instead of 4, and with a ring half as deep the gate/up kernel fits three waves per SIMD instead of two, which hides
// some of the decode's latency (an LDS table read, then a chain of byte permutes): about 1 us of the 33 the launch
// took on the 32-token layer of 65 slots.  A deeper ring (8, or 8 in the down pass) and two stripes per wave in the
// down pass measured slower.  The bf16 cases of this kernel (an expert stored raw) use the same parameters.
constexpr int kP12RT0 = 2, kP12D0 = 4;
constexpr int kP12RT1 = 4, kP12D1 = 4;
template <int PASS, bool P12SLOTS>
constexpr int small_rt() { return P12SLOTS ? (PASS == 0 ? kP12RT0 : kP12RT1) : (PASS == 0 ? kSmallRT0 : kSmallRT1); }
template <int PASS, bool P12SLOTS>
constexpr int small_depth() { return P12SLOTS ? (PASS == 0 ? kP12D0 : kP12D1) : (PASS == 0 ? kSmallD0 : kSmallD1); }
template <int PASS, bool P12SLOTS>
__global__ __launch_bounds__(kWaves * 64) void expert_gemm_kernel(
    const uint16_t* __restrict__ slots, int64_t blob_elems, int64_t off_w,
    const Task* __restrict__ tasks, const int32_t* __restrict__ n_tasks, const uint16_t* __restrict__ act_in,
    const int32_t* __restrict__ row_token, int K, int n_out, uint16_t* __restrict__ act_out,
    float* __restrict__ y_out) {
    constexpr int RT = small_rt<PASS, P12SLOTS>();
    constexpr int D = small_depth<PASS, P12SLOTS>();
    __shared__ __attribute__((aligned(16))) uint16_t lds[kRowsPerTask * (kSmallPC * 32 + 8)];
    __shared__ uint4 tables[P12SLOTS ? kWaves : 1][64];     // 12-bit slots: each wave's tile tables
    const int task_id = blockIdx.y;
    if (task_id >= n_tasks[0]) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // the same for a wave's lanes: scalar
    const int wtile = blockIdx.x * kWaves + wave;
    const bool active = wtile * 16 * (PASS == 0 ? RT / 2 : RT) < n_out;      // spare waves still help staging
    const Task task = tasks[task_id];
    const uint16_t* blob = slots + (int64_t)task.slot * blob_elems;
    static_assert(kRowsPerTask == 32, "one or two 16-token tiles per small work item");
    // sibling items of one slot (kTaskSiblings) use cacheable weight loads; up to 16 rows take one token tile
#define TIDE_SMALL_CASE(NT_, SIB_, FMT_)                                                                                 \
    gemm_task<PASS, RT, NT_, D, kSmallPC, 1, SIB_, FMT_>(blob, off_w, wtile, active, task, act_in, row_token, K, n_out, \
                                                        blob_elems, act_out, y_out, lds, tables[P12SLOTS ? wave : 0])
    const bool one = task.nrows <= 16;
    // a context with bf16 slots never flags a work item kTaskP12: those cases are not compiled into its kernel
    const int flags = task.flags & (P12SLOTS ? (kTaskSiblings | kTaskP12) : kTaskSiblings);
    if (flags == 0) {
        if (one) TIDE_SMALL_CASE(1, false, kFmtBf16); else TIDE_SMALL_CASE(2, false, kFmtBf16);
    } else if (flags == kTaskSiblings) {
        if (one) TIDE_SMALL_CASE(1, true, kFmtBf16); else TIDE_SMALL_CASE(2, true, kFmtBf16);
    } else if constexpr (P12SLOTS) {
        if (flags == kTaskP12) {
            if (one) TIDE_SMALL_CASE(1, false, kFmtP12); else TIDE_SMALL_CASE(2, false, kFmtP12);
        } else {
            if (one) TIDE_SMALL_CASE(1, true, kFmtP12); else TIDE_SMALL_CASE(2, true, kFmtP12);
        }
    }
#undef TIDE_SMALL_CASE
}

// Large work items: up to 256 rows of a slot that holds more than 32.  A workgroup's tile is 256
// weight rows x up to 256 tokens: what bounds these kernels is the rate at which a compute unit's
// vector cache can be filled, so the tile is as large as the accumulators allow (256 of a wave's 512
// registers).  Up to 128 rows: eight token tiles, 256-column stages.  Above: up to 16 token tiles in two
// half sets, 128-column stages.  Ring depth 4 for both: a deeper ring reads no faster (a read-only kernel
// with this access shape and one workgroup per compute unit is slower at depth 8 than at 4) and measured
// 1-3 % slower in the step.
constexpr int kBigPC = 8, kBigD = 4;       // <= 8 token tiles
constexpr int kWidePC = 4, kWideD = 4;     // 9..16 token tiles
constexpr int kBigPC12 = 4, kWidePC12 = 2; // the stages over a 12-bit slot (<= 8, 9..12 token tiles)
constexpr int kBigLdsElems = 2 * 128 * (kBigPC * 32 + 8) > 2 * 256 * (kWidePC * 32 + 8) ? 2 * 128 * (kBigPC * 32 + 8)
                                                                                      : 2 * 256 * (kWidePC * 32 + 8);
constexpr int kXcds = 8;           // accelerator complex dies, each with its own L2

// Order of the large work.  The work items are ranked heaviest first (plan_big_kernel) and dealt to
// eight lists, one per XCD, in serpentine order (ranks 0..7 to lists 0..7, ranks 8..15 to lists 7..0,
// ...), so the lists hold about equal work.  Workgroups are handed to the XCDs round-robin by linear
// id and started in id order as compute units fall free: workgroup b runs on XCD b % 8 and takes unit
// b / 8 of that XCD's list (its work items in rank order, feature tile fastest).  Heavy units start
// first, the light ones fill the end of the launch; the units of a work item share their token rows
// through the XCD's L2.
__device__ inline int list_tasks(int x, int n) {         // work items in list x when n are ranked
    const int lo = x, hi = 2 * kXcds - 1 - x;
    return (n > lo ? (n - lo + 2 * kXcds - 1) / (2 * kXcds) : 0) + (n > hi ? (n - hi + 2 * kXcds - 1) / (2 * kXcds) : 0);
}
__device__ inline int list_rank(int x, int j) {          // rank of list x's j-th work item
    return (j >> 1) * 2 * kXcds + ((j & 1) ? 2 * kXcds - 1 - x : x);
}

constexpr int kPlanThreads = 256;
constexpr int kTileClasses = kRowsPerBigTask / 16;       // work items are ranked by their number of 16-token tiles
__global__ __launch_bounds__(kPlanThreads) void plan_big_kernel(const Task* __restrict__ tasks,
                                                               const int32_t* __restrict__ n_tasks,
                                                               int32_t* __restrict__ order) {
    __shared__ int count[kTileClasses + 1], first[kTileClasses + 1];
    const int tid = threadIdx.x, n = n_tasks[1];
    if (tid <= kTileClasses) count[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kPlanThreads) atomicAdd(&count[min((tasks[i].nrows + 15) >> 4, kTileClasses)], 1);
    __syncthreads();
    if (tid == 0) {
        int at = 0;
        for (int c = kTileClasses; c >= 0; --c) {
            first[c] = at;
            at += count[c];
        }
    }
    __syncthreads();
    // the order inside a class does not matter (equal cost); every rank 0..n-1 is written exactly once
    for (int i = tid; i < n; i += kPlanThreads) order[atomicAdd(&first[min((tasks[i].nrows + 15) >> 4, kTileClasses)], 1)] = i;
}

template <int PASS>
__global__ __launch_bounds__(kWaves * 64) void expert_gemm_big_kernel(
    const uint16_t* __restrict__ slots, int64_t blob_elems, int64_t off_w, const Task* __restrict__ tasks,
    const int32_t* __restrict__ n_tasks, const int32_t* __restrict__ order, const uint16_t* __restrict__ act_in,
    const int32_t* __restrict__ row_token, int K, int n_out, uint16_t* __restrict__ act_out,
    float* __restrict__ y_out, int n_ftiles) {
    constexpr int RT = 4;
    __shared__ __attribute__((aligned(16))) uint16_t lds[kBigLdsElems];
    __shared__ uint4 tables[kWaves][2 * 64];           // 12-bit slots: each wave's tile tables, two blocks of them
    const int n_big = n_tasks[1];
    const int xcd = blockIdx.x % kXcds, unit = blockIdx.x / kXcds;
    if (unit >= list_tasks(xcd, n_big) * n_ftiles) return;
    const int task_id = order[list_rank(xcd, unit / n_ftiles)];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // scalar, as above
    const int wtile = (unit % n_ftiles) * kWaves + wave;
    const bool active = wtile * 16 * (PASS == 0 ? RT / 2 : RT) < n_out;
    const Task task = tasks[task_id];
    const uint16_t* blob = slots + (int64_t)task.slot * blob_elems;
    static_assert(kRowsPerBigTask == 256, "sixteen 16-token tiles per large work item");
    // only as many 16-token tiles as the item has rows: a 40-row item costs 3/8 of a 128-row one
#define TIDE_BIG_CASE(NT_)                                                                                              \
    case NT_:                                                                                                           \
        gemm_task<PASS, RT, NT_, kBigD, BPC, 2, false, FMT>(blob, off_w, wtile, active, task, act_in, row_token, K,      \
                                                            n_out, blob_elems, act_out, y_out, lds, tables[wave]);     \
        break;
#define TIDE_WIDE_CASE(NT_)                                                                                             \
    case NT_ - 1:                                                                                                       \
    case NT_:                                                                                                           \
        gemm_task<PASS, RT, NT_, kWideD, WPC, 2, false, FMT>(blob, off_w, wtile, active, task, act_in, row_token, K,     \
                                                             n_out, blob_elems, act_out, y_out, lds, tables[wave]);    \
        break;
    auto run = [&](auto fmt) {
        constexpr int FMT = decltype(fmt)::value;
        // 12-bit slots: the decode's registers come out of the token staging (stages half as wide), and a work item
        // has at most kRowsPerBigTaskP12 rows
        constexpr int BPC = FMT == kFmtP12 ? kBigPC12 : kBigPC;
        constexpr int WPC = FMT == kFmtP12 ? kWidePC12 : kWidePC;
        static_assert(kRowsPerBigTaskP12 == 192, "twelve 16-token tiles per large work item over a 12-bit slot");
        switch ((task.nrows + 15) >> 4) {
            TIDE_BIG_CASE(1) TIDE_BIG_CASE(2) TIDE_BIG_CASE(3) TIDE_BIG_CASE(4) TIDE_BIG_CASE(5) TIDE_BIG_CASE(6) TIDE_BIG_CASE(7)
            TIDE_BIG_CASE(8) TIDE_WIDE_CASE(10) TIDE_WIDE_CASE(12)
            default:
                if constexpr (FMT == kFmtBf16) {
                    if (task.nrows <= 14 * 16)
                        gemm_task<PASS, RT, 14, kWideD, WPC, 2, false, FMT>(blob, off_w, wtile, active, task, act_in, row_token, K,
                                                                            n_out, blob_elems, act_out, y_out, lds, tables[wave]);
                    else
                        gemm_task<PASS, RT, 16, kWideD, WPC, 2, false, FMT>(blob, off_w, wtile, active, task, act_in, row_token, K,
                                                                            n_out, blob_elems, act_out, y_out, lds, tables[wave]);
                }
        }
    };
    if (task.flags & kTaskP12) run(std::integral_constant<int, kFmtP12>{});
    else run(std::integral_constant<int, kFmtBf16>{});
#undef TIDE_BIG_CASE
#undef TIDE_WIDE_CASE
}

}  // namespace

hipError_t launch_expert_gemm(int pass, const Shape& s, const LayerTables& t, const Workspace& w, const uint16_t* x,
                              int max_tasks, hipStream_t stream, LaunchEvents ev) {
    if (max_tasks <= 0) return hipSuccess;
    dim3 block(kWaves * 64);
    auto launch = [&](auto p12) {
        constexpr bool P12 = decltype(p12)::value;
        if (pass == 0) {
            constexpr int cols = 16 * kWaves * (small_rt<0, P12>() / 2);      // SwiGLU columns per workgroup
            TIDE_LAUNCH((expert_gemm_kernel<0, P12>), dim3((s.I + cols - 1) / cols, max_tasks), block, stream, ev, t.slots, s.blob_elems,
                        blob_off_gate_up(s), w.tasks, w.n_tasks, x, w.row_token, s.d, s.I, w.act,
                        (float*)nullptr);
        } else {
            constexpr int cols = 16 * kWaves * small_rt<1, P12>();            // output columns per workgroup
            TIDE_LAUNCH((expert_gemm_kernel<1, P12>), dim3((s.d + cols - 1) / cols, max_tasks), block, stream, ev, t.slots, s.blob_elems,
                        blob_off_down(s), w.tasks, w.n_tasks, w.act, w.row_token, s.I, s.d,
                        (uint16_t*)nullptr, w.y);
        }
    };
    // the miss pass reads the host's bf16 blobs through a table view without format flags: the bf16 kernel
    if (t.expert_p12) launch(std::true_type{});
    else launch(std::false_type{});
    return hipGetLastError();
}

hipError_t launch_plan_big(const Workspace& w, int max_big_tasks, hipStream_t stream) {
    if (max_big_tasks <= 0) return hipSuccess;
    hipLaunchKernelGGL(plan_big_kernel, dim3(1), dim3(kPlanThreads), 0, stream, w.big_tasks, w.n_tasks, w.big_order);
    return hipGetLastError();
}

hipError_t launch_expert_gemm_big(int pass, const Shape& s, const LayerTables& t, const Workspace& w,
                                  const uint16_t* x, int max_big_tasks, hipStream_t stream, LaunchEvents ev) {
    if (max_big_tasks <= 0) return hipSuccess;
    dim3 block(kWaves * 64);
    const int ft = pass == 0 ? (s.I + 127) / 128 : (s.d + 255) / 256;
    // the longest list holds 2 * ceil(n / 16) work items
    const dim3 grid((unsigned)((max_big_tasks + 2 * kXcds - 1) / (2 * kXcds) * 2 * ft * kXcds));
    if (pass == 0) {
        TIDE_LAUNCH(expert_gemm_big_kernel<0>, grid, block, stream, ev, t.slots, s.blob_elems, blob_off_gate_up(s),
                    w.big_tasks, w.n_tasks, w.big_order, x, w.row_token, s.d, s.I, w.act, (float*)nullptr, ft);
    } else {
        TIDE_LAUNCH(expert_gemm_big_kernel<1>, grid, block, stream, ev, t.slots, s.blob_elems, blob_off_down(s),
                    w.big_tasks, w.n_tasks, w.big_order, w.act, w.row_token, s.I, s.d, (uint16_t*)nullptr, w.y, ft);
    }
    return hipGetLastError();
}

}  // namespace tide
