// Host-core execution of missed experts (Sec. 3.3, Alg. 1: a token whose expert is not in the
// GPU set is evaluated by the CPU copy of that expert, concurrently with the GPU's hits).
//
// The worker threads read the packed blobs exactly as they lie in pinned host memory: 16-row x
// 32-column tiles, lane-major, i.e. a tile is 64 pieces of 8 consecutive K elements of one row
// (piece (q*16 + r) = row r, K offset q*8).  A piece is one 8-wide vector: it is multiplied with
// the 8 matching elements of a token row and added into an 8-wide accumulator per (token, weight
// row); the accumulators of one stripe group live in the core's L1 while the group's region of the
// blob is streamed front to back once, and are summed across their 8 lanes at the end.
// On cores with AVX-512 BF16 the same walk uses the bf16 dot-product instruction instead: a 64-byte line of
// a tile is four rows x 8 K elements, one instruction multiplies it with a token's 8 bf16 elements (no
// conversion of either operand) and adds the products pairwise into 16 fp32 lanes, four per row.
#include "host_experts.h"

#include <immintrin.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace tide {

namespace {

typedef float f8 __attribute__((vector_size(32)));
typedef uint16_t h8 __attribute__((vector_size(16)));
typedef uint32_t w8 __attribute__((vector_size(32)));

constexpr int kTokBlock = 4;                  // tokens whose accumulators are live together
constexpr int kAccRows = 256;                 // weight rows of a stripe group (gate + up, or 16 down stripes)

#define TIDE_INLINE inline __attribute__((always_inline))

TIDE_INLINE f8 bf16x8(const uint16_t* p) {
    h8 v;
    memcpy(&v, p, 16);
    w8 w = __builtin_convertvector(v, w8) << 16;
    f8 f;
    memcpy(&f, &w, 32);
    return f;
}
TIDE_INLINE f8 ldf8(const float* p) {
    f8 v;
    memcpy(&v, p, 32);
    return v;
}
// fp32 -> nearest bf16 (ties to even) -> fp32: the intermediate activation is stored in bf16, as on the GPU
TIDE_INLINE float round_bf16(float v) {
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&v, &u, 4);
    return v;
}
TIDE_INLINE float hsum(f8 v) { return ((v[0] + v[4]) + (v[2] + v[6])) + ((v[1] + v[5]) + (v[3] + v[7])); }

struct PartArgs {
    const uint16_t* blob;
    int d, d_ff;
    int g0, g1;               // gate/up groups [g0, g1) of the expert: columns g*128.. of the intermediate
    int m;                    // tokens
    const float* const* x;    // m pointers to fp32 token rows [d] (vector path)
    const uint16_t* const* xb;  // m pointers to bf16 token rows [d] (bf16 dot-product path)
    float* y;                 // [m][d], overwritten: the part of e(x) that comes from those columns
    f8* acc;                  // [kTokBlock][kAccRows] scratch, 64-byte aligned
    float* h;                 // [kTokBlock][128] scratch (the bf16 path keeps bf16 bits in its first half)
};

// acc[t][j*16 + r] += tile piece (q, r) * operand piece q of token t, over `ntiles` consecutive tiles
template <int TB>
TIDE_INLINE void tiles_fma(const uint16_t* tiles, int ntiles, const f8 (&xq)[4][kTokBlock], f8* acc, int acc_stride) {
    for (int j = 0; j < ntiles; ++j) {
        const uint16_t* tp = tiles + j * 512;
        for (int r = 0; r < 16; ++r) {
            f8 a[TB];
            for (int t = 0; t < TB; ++t) a[t] = acc[t * acc_stride + j * 16 + r];
            for (int q = 0; q < 4; ++q) {
                const f8 w = bf16x8(tp + (q * 16 + r) * 8);
                for (int t = 0; t < TB; ++t) a[t] += w * xq[q][t];
            }
            for (int t = 0; t < TB; ++t) acc[t * acc_stride + j * 16 + r] = a[t];
        }
    }
}

// one gate/up group g (128 columns of the intermediate) for TB tokens: y[t0..][:] += their part of e(x)
template <int TB>
TIDE_INLINE void part_block(const PartArgs& a, int g, int t0) {
    const int d = a.d, I = a.d_ff, kcd = d / 32, kci = I / 32, blocks = I / 16, stripes = d / 16;
    const uint16_t* down = a.blob + 2ll * d * I;
    {
        const int ng = std::min(kHostGateUpGroup, blocks - g * kHostGateUpGroup);
        const int rows = 2 * ng * 16;
        for (int i = 0; i < TB * rows; ++i) a.acc[i] = f8{0, 0, 0, 0, 0, 0, 0, 0};
        const uint16_t* base = a.blob + (int64_t)g * 2 * kHostGateUpGroup * kcd * 512;
        for (int kc = 0; kc < kcd; ++kc) {
            f8 xq[4][kTokBlock];
            for (int q = 0; q < 4; ++q)
                for (int t = 0; t < TB; ++t) xq[q][t] = ldf8(a.x[t0 + t] + kc * 32 + q * 8);
            tiles_fma<TB>(base + (int64_t)kc * 2 * ng * 512, 2 * ng, xq, a.acc, rows);
        }
        // SwiGLU: columns g*128 + c of the intermediate (gate rows first, then the up rows)
        const int ncol = ng * 16;
        for (int t = 0; t < TB; ++t)
            for (int c = 0; c < ncol; ++c) {
                const float gate = hsum(a.acc[t * rows + c]), up = hsum(a.acc[t * rows + ncol + c]);
                a.h[t * 128 + c] = round_bf16(gate / (1.0f + expf(-gate)) * up);
            }
        // down projection of those columns: K chunks g*4 .. of every down stripe group
        const int nkc = ncol / 32;
        for (int G = 0; G * kHostDownGroup < stripes; ++G) {
            const int ngd = std::min(kHostDownGroup, stripes - G * kHostDownGroup);
            const int drows = ngd * 16;
            for (int i = 0; i < TB * drows; ++i) a.acc[i] = f8{0, 0, 0, 0, 0, 0, 0, 0};
            const uint16_t* gbase = down + (int64_t)G * kHostDownGroup * kci * 512;
            for (int kk = 0; kk < nkc; ++kk) {
                const int kc = g * (kHostGateUpGroup / 2) + kk;
                f8 hq[4][kTokBlock];
                for (int q = 0; q < 4; ++q)
                    for (int t = 0; t < TB; ++t) hq[q][t] = ldf8(a.h + t * 128 + kk * 32 + q * 8);
                tiles_fma<TB>(gbase + (int64_t)kc * ngd * 512, ngd, hq, a.acc, drows);
            }
            for (int t = 0; t < TB; ++t) {
                float* yr = a.y + (int64_t)(t0 + t) * d + G * kHostDownGroup * 16;
                for (int c = 0; c < drows; ++c) yr[c] += hsum(a.acc[t * drows + c]);
            }
        }
    }
}

// Group by group, every token block inside: a group's region of the blob (gate/up stripes and the matching K
// chunks of the down stripes) comes from memory once and from the core's caches for the later token blocks.
TIDE_INLINE void part_body(const PartArgs& a) {
    memset(a.y, 0, sizeof(float) * (size_t)a.m * a.d);
    for (int g = a.g0; g < a.g1; ++g)
        for (int t0 = 0; t0 < a.m; t0 += kTokBlock) {
            switch (std::min(kTokBlock, a.m - t0)) {
                case 1: part_block<1>(a, g, t0); break;
                case 2: part_block<2>(a, g, t0); break;
                case 3: part_block<3>(a, g, t0); break;
                default: part_block<4>(a, g, t0); break;
            }
        }
}

__attribute__((target("avx2,fma"))) void part_avx2(const PartArgs& a) { part_body(a); }
void part_generic(const PartArgs& a) { part_body(a); }

// ---- AVX-512 BF16 ------------------------------------------------------------------------------------
#define TIDE_BF16 __attribute__((target("avx512f,avx512bw,avx512vl,avx512bf16")))
#define TIDE_BF16_INLINE TIDE_BF16 inline __attribute__((always_inline))

TIDE_BF16_INLINE uint16_t bf16_bits(float v) {
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// acc[t][j*4 + rr] (16 lanes: rows rr*4 .. +3 of tile j, four partial sums each) += line (q, rr) of the tile
// dotted pairwise with the 8 bf16 operand elements of token t at K offset q*8
template <int TB>
TIDE_BF16_INLINE void tiles_dp(const uint16_t* tiles, int ntiles, const uint16_t* const (&xk)[kTokBlock], __m512* acc,
                               int acc_stride) {
    for (int j = 0; j < ntiles; ++j) {
        const char* tp = reinterpret_cast<const char*>(tiles + j * 512);
        __m512 a[TB][4];
        for (int t = 0; t < TB; ++t)
            for (int rr = 0; rr < 4; ++rr) a[t][rr] = acc[t * acc_stride + j * 4 + rr];
        for (int q = 0; q < 4; ++q) {
            __m512bh xq[TB];
            for (int t = 0; t < TB; ++t)
                xq[t] = (__m512bh)_mm512_broadcast_i32x4(_mm_loadu_si128(reinterpret_cast<const __m128i*>(xk[t] + q * 8)));
            for (int rr = 0; rr < 4; ++rr) {
                const __m512bh w = (__m512bh)_mm512_loadu_si512(tp + (q * 4 + rr) * 64);
                for (int t = 0; t < TB; ++t) a[t][rr] = _mm512_dpbf16_ps(a[t][rr], w, xq[t]);
            }
        }
        for (int t = 0; t < TB; ++t)
            for (int rr = 0; rr < 4; ++rr) acc[t * acc_stride + j * 4 + rr] = a[t][rr];
    }
}

// sum of the four partial lanes of row c (lanes 4*(c%4) .. +3 of accumulator c/4)
TIDE_BF16_INLINE float row_sum(const float* acc_f, int c) {
    const float* p = acc_f + (c >> 2) * 16 + (c & 3) * 4;
    return (p[0] + p[2]) + (p[1] + p[3]);
}

template <int TB>
TIDE_BF16_INLINE void part_block_bf16(const PartArgs& a, int g, int t0) {
    const int d = a.d, I = a.d_ff, kcd = d / 32, kci = I / 32, blocks = I / 16, stripes = d / 16;
    const uint16_t* down = a.blob + 2ll * d * I;
    __m512* acc = reinterpret_cast<__m512*>(a.acc);
    const float* acc_f = reinterpret_cast<const float*>(a.acc);
    uint16_t* h16 = reinterpret_cast<uint16_t*>(a.h);                 // [TB][128] bf16 bits
    {
        const int ng = std::min(kHostGateUpGroup, blocks - g * kHostGateUpGroup);
        const int rows = 2 * ng * 16, stride = rows / 4;
        for (int i = 0; i < TB * stride; ++i) acc[i] = _mm512_setzero_ps();
        const uint16_t* base = a.blob + (int64_t)g * 2 * kHostGateUpGroup * kcd * 512;
        for (int kc = 0; kc < kcd; ++kc) {
            const uint16_t* xk[kTokBlock];
            for (int t = 0; t < TB; ++t) xk[t] = a.xb[t0 + t] + kc * 32;
            tiles_dp<TB>(base + (int64_t)kc * 2 * ng * 512, 2 * ng, xk, acc, stride);
        }
        const int ncol = ng * 16;
        for (int t = 0; t < TB; ++t)
            for (int c = 0; c < ncol; ++c) {
                const float gate = row_sum(acc_f + t * rows * 4, c), up = row_sum(acc_f + t * rows * 4, ncol + c);
                h16[t * 128 + c] = bf16_bits(gate / (1.0f + expf(-gate)) * up);
            }
        const int nkc = ncol / 32;
        for (int G = 0; G * kHostDownGroup < stripes; ++G) {
            const int ngd = std::min(kHostDownGroup, stripes - G * kHostDownGroup);
            const int drows = ngd * 16, dstride = drows / 4;
            for (int i = 0; i < TB * dstride; ++i) acc[i] = _mm512_setzero_ps();
            const uint16_t* gbase = down + (int64_t)G * kHostDownGroup * kci * 512;
            for (int kk = 0; kk < nkc; ++kk) {
                const int kc = g * (kHostGateUpGroup / 2) + kk;
                const uint16_t* hk[kTokBlock];
                for (int t = 0; t < TB; ++t) hk[t] = h16 + t * 128 + kk * 32;
                tiles_dp<TB>(gbase + (int64_t)kc * ngd * 512, ngd, hk, acc, dstride);
            }
            for (int t = 0; t < TB; ++t) {
                float* yr = a.y + (int64_t)(t0 + t) * d + G * kHostDownGroup * 16;
                for (int c = 0; c < drows; ++c) yr[c] += row_sum(acc_f + t * drows * 4, c);
            }
        }
    }
}

TIDE_BF16 void part_bf16(const PartArgs& a) {
    memset(a.y, 0, sizeof(float) * (size_t)a.m * a.d);
    for (int g = a.g0; g < a.g1; ++g)
        for (int t0 = 0; t0 < a.m; t0 += kTokBlock) {
            switch (std::min(kTokBlock, a.m - t0)) {
                case 1: part_block_bf16<1>(a, g, t0); break;
                case 2: part_block_bf16<2>(a, g, t0); break;
                case 3: part_block_bf16<3>(a, g, t0); break;
                default: part_block_bf16<4>(a, g, t0); break;
            }
        }
}

enum Isa { kGeneric = 0, kAvx2 = 1, kAvx512Bf16 = 2 };
Isa detect_isa() {
    const char* force = getenv("TIDE_HOST_ISA");              // "generic" | "avx2": for checking the other paths
    __builtin_cpu_init();
    const bool avx2 = __builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma");
    const bool bf16 = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
                      __builtin_cpu_supports("avx512vl") && __builtin_cpu_supports("avx512bf16");
    if (force && !strcmp(force, "generic")) return kGeneric;
    if (force && !strcmp(force, "avx2")) return avx2 ? kAvx2 : kGeneric;
    return bf16 ? kAvx512Bf16 : avx2 ? kAvx2 : kGeneric;
}

Isa host_isa() {
    static const Isa isa = detect_isa();
    return isa;
}

void run_part(const PartArgs& a) {
    const Isa isa = host_isa();
    if (isa == kAvx512Bf16) part_bf16(a);
    else if (isa == kAvx2) part_avx2(a);
    else part_generic(a);
}

struct Scratch {
    f8* acc = nullptr;
    float* h = nullptr;
    Scratch() {
        acc = static_cast<f8*>(aligned_alloc(64, sizeof(f8) * kTokBlock * kAccRows));
        h = static_cast<float*>(aligned_alloc(64, sizeof(float) * kTokBlock * 128));
    }
    ~Scratch() { free(acc); free(h); }
    Scratch(const Scratch&) = delete;
    Scratch& operator=(const Scratch&) = delete;
};

void bf16_row_to_f32(const uint16_t* src, float* dst, int n) {
    for (int i = 0; i < n; ++i) {
        const uint32_t u = (uint32_t)src[i] << 16;
        memcpy(dst + i, &u, 4);
    }
}

}  // namespace

struct HostPool {
    int n = 1;
    std::vector<std::thread> workers;
    std::vector<Scratch> scratch;
    std::mutex mu;
    std::condition_variable cv_go, cv_done;
    uint64_t gen = 0;
    bool stop = false;
    const std::function<void(int, int)>* fn = nullptr;
    int n_tasks = 0;
    std::atomic<int> next{0};
    int running = 0;
    // buffers reused from call to call
    std::vector<float> xf, ypart;
    std::vector<const float*> xptr;
    std::vector<const uint16_t*> xbptr;
    std::vector<int32_t> by_expert, pos_of, exp_off, tok_off, by_token, tok_row;
    std::vector<tide_miss> kept;

    explicit HostPool(int threads) : n(threads), scratch(threads) {}

    void work(int id) {
        for (;;) {
            const int t = next.fetch_add(1, std::memory_order_relaxed);
            if (t >= n_tasks) break;
            (*fn)(t, id);
        }
    }
    void loop(int id) {
        uint64_t seen = 0;
        std::unique_lock<std::mutex> lk(mu);
        for (;;) {
            cv_go.wait(lk, [&] { return stop || gen != seen; });
            if (stop) return;
            seen = gen;
            lk.unlock();
            work(id);
            lk.lock();
            if (--running == 0) cv_done.notify_one();
        }
    }
    // fn(task, worker) for task in [0, tasks), spread over the threads; returns when all are done
    void run(int tasks, const std::function<void(int, int)>& f) {
        if (tasks <= 0) return;
        {
            std::lock_guard<std::mutex> lk(mu);
            fn = &f;
            n_tasks = tasks;
            next.store(0, std::memory_order_relaxed);
            running = (int)workers.size();
            ++gen;
        }
        cv_go.notify_all();
        work(0);
        std::unique_lock<std::mutex> lk(mu);
        cv_done.wait(lk, [&] { return running == 0; });
    }
};

HostPool* host_pool_create(int n_threads) {
    if (n_threads < 1) n_threads = 1;
    HostPool* p = new HostPool(n_threads);
    for (int i = 1; i < n_threads; ++i) p->workers.emplace_back([p, i] { p->loop(i); });
    return p;
}

void host_pool_destroy(HostPool* p) {
    if (!p) return;
    {
        std::lock_guard<std::mutex> lk(p->mu);
        p->stop = true;
    }
    p->cv_go.notify_all();
    for (std::thread& t : p->workers) t.join();
    delete p;
}

int host_pool_threads(const HostPool* p) { return p ? p->n : 0; }

void host_expert_forward(const void* blob, int d, int d_ff, const uint16_t* x, int m, float* y) {
    Scratch s;
    std::vector<float> xf((size_t)m * d);
    std::vector<const float*> xp(m);
    std::vector<const uint16_t*> xbp(m);
    for (int t = 0; t < m; ++t) {
        if (host_isa() != kAvx512Bf16) bf16_row_to_f32(x + (int64_t)t * d, xf.data() + (int64_t)t * d, d);
        xp[t] = xf.data() + (int64_t)t * d;
        xbp[t] = x + (int64_t)t * d;
    }
    const int groups = (d_ff / 16 + kHostGateUpGroup - 1) / kHostGateUpGroup;
    PartArgs a{static_cast<const uint16_t*>(blob), d, d_ff, 0, groups, m, xp.data(), xbp.data(), y, s.acc, s.h};
    run_part(a);
}

int host_apply_misses(HostPool* p, const uint8_t* blobs, uint64_t stride, int d, int d_ff, int n_experts,
                      const uint16_t* x, int n_tokens, const tide_miss* miss_all, int n_all, float* y_rows,
                      int32_t* tokens_out, const uint8_t* skip_expert) {
    if (n_all <= 0) return 0;
    for (int i = 0; i < n_all; ++i)
        if (miss_all[i].token < 0 || miss_all[i].token >= n_tokens || miss_all[i].expert < 0 || miss_all[i].expert >= n_experts)
            return -1;
    // the entries this call evaluates, in list order
    const tide_miss* miss = miss_all;
    int n = n_all;
    if (skip_expert) {
        p->kept.clear();
        for (int i = 0; i < n_all; ++i)
            if (!skip_expert[miss_all[i].expert]) p->kept.push_back(miss_all[i]);
        miss = p->kept.data();
        n = (int)p->kept.size();
        if (n == 0) return 0;
    }
    // the list grouped by expert (stable) and by token (stable: list order inside a token)
    p->exp_off.assign(n_experts + 1, 0);
    p->tok_off.assign(n_tokens + 1, 0);
    for (int i = 0; i < n; ++i) {
        p->exp_off[miss[i].expert + 1]++;
        p->tok_off[miss[i].token + 1]++;
    }
    for (int e = 0; e < n_experts; ++e) p->exp_off[e + 1] += p->exp_off[e];
    for (int t = 0; t < n_tokens; ++t) p->tok_off[t + 1] += p->tok_off[t];
    p->by_expert.resize(n);
    p->by_token.resize(n);
    p->pos_of.resize(n);
    {
        std::vector<int32_t> ce(p->exp_off.begin(), p->exp_off.end() - 1), ct(p->tok_off.begin(), p->tok_off.end() - 1);
        for (int i = 0; i < n; ++i) {
            p->pos_of[i] = ce[miss[i].expert];
            p->by_expert[ce[miss[i].expert]++] = i;
            p->by_token[ct[miss[i].token]++] = i;
        }
    }
    // rows of the result: the tokens with at least one miss, ascending
    p->tok_row.assign(n_tokens, -1);
    int n_rows = 0;
    for (int t = 0; t < n_tokens; ++t)
        if (p->tok_off[t + 1] > p->tok_off[t]) {
            p->tok_row[t] = n_rows;
            tokens_out[n_rows++] = t;
        }
    // fp32 copies of those tokens' states
    p->xf.resize((size_t)n_rows * d);
    float* xf = p->xf.data();
    if (host_isa() != kAvx512Bf16)          // the bf16 dot-product path reads the token states as they are
        p->run(n_rows, [&](int r, int) { bf16_row_to_f32(x + (int64_t)tokens_out[r] * d, xf + (int64_t)r * d, d); });
    p->xptr.resize(n);
    p->xbptr.resize(n);
    for (int j = 0; j < n; ++j) {
        const int tok = miss[p->by_expert[j]].token;
        p->xptr[j] = xf + (int64_t)p->tok_row[tok] * d;
        p->xbptr[j] = x + (int64_t)tok * d;
    }

    // work items: (expert with misses, part of its intermediate columns).  With few missed experts each is
    // cut into its gate/up groups so that every core has work; otherwise one item per expert.
    std::vector<int32_t> experts;
    for (int e = 0; e < n_experts; ++e)
        if (p->exp_off[e + 1] > p->exp_off[e]) experts.push_back(e);
    std::stable_sort(experts.begin(), experts.end(), [&](int a, int b) {
        return p->exp_off[a + 1] - p->exp_off[a] > p->exp_off[b + 1] - p->exp_off[b]; });
    const int groups = (d_ff / 16 + kHostGateUpGroup - 1) / kHostGateUpGroup;
    const int parts = ((int)experts.size() >= 4 * p->n) ? 1 : groups;
    const int per_part = (groups + parts - 1) / parts;
    p->ypart.resize((size_t)parts * n * d);
    float* ypart = p->ypart.data();
    const int n_items = (int)experts.size() * parts;
    p->run(n_items, [&](int item, int worker) {
        const int e = experts[item / parts], part = item % parts;
        const int j0 = p->exp_off[e], m = p->exp_off[e + 1] - j0;
        PartArgs a{reinterpret_cast<const uint16_t*>(blobs + (uint64_t)e * stride), d, d_ff, part * per_part,
                   std::min(groups, (part + 1) * per_part), m, p->xptr.data() + j0, p->xbptr.data() + j0,
                   ypart + ((int64_t)part * n + j0) * d, p->scratch[worker].acc, p->scratch[worker].h};
        run_part(a);
    });
    // per token: weighted sum of its misses in list order, the parts of an expert in column order
    p->run(n_rows, [&](int r, int) {
        const int t = tokens_out[r];
        float* yr = y_rows + (int64_t)r * d;
        memset(yr, 0, sizeof(float) * d);
        for (int q = p->tok_off[t]; q < p->tok_off[t + 1]; ++q) {
            const int i = p->by_token[q];
            const float w = miss[i].weight;
            const float* src = ypart + (int64_t)p->pos_of[i] * d;
            for (int c = 0; c < d; ++c) {
                float s = src[c];
                for (int part = 1; part < parts; ++part) s += src[(int64_t)part * n * d + c];
                yr[c] += w * s;
            }
        }
    });
    return n_rows;
}

}  // namespace tide
