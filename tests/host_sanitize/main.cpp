// Host-side parts of libtide under the sanitizers: expert packing, the 12-bit form, one expert on the calling
// thread, and the worker pool's miss pass.  Built by tests/test_host_sanitizers.py from the library's own
// host-only sources with -fsanitize=address,undefined or -fsanitize=thread; exits non-zero on any wrong result
// (the sanitizers abort on their own findings).
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "host_experts.h"
#include "host_pack.h"
#include "packed12.h"

using namespace tide;

static uint32_t rng_state = 12345u;
static uint32_t next_u32() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state; }
static float next_unit() { return (float)(next_u32() >> 8) / 16777216.0f - 0.5f; }
static uint16_t bf16_of(float f) { uint32_t u; memcpy(&u, &f, 4); u += 0x7FFFu + ((u >> 16) & 1u); return (uint16_t)(u >> 16); }
static float f32_of(uint16_t b) { uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4); return f; }

#define CHECK(cond)                                                             \
    do {                                                                        \
        if (!(cond)) { fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); exit(1); } \
    } while (0)

// decoder written from the format's description: a lane's two dwords of low bytes and its dword of 4-bit table
// indices, the tile's table of high bytes (tables are stored stripe first inside a stripe group)
static std::vector<uint16_t> decode_p12(const std::vector<uint8_t>& comp, uint64_t blob_bytes, int d, int d_ff) {
    const uint32_t n_tiles = (uint32_t)(blob_bytes / 1024);
    const P12Layout lay = p12_layout(n_tiles);
    std::vector<uint16_t> out(blob_bytes / 2);
    for (uint32_t t = 0; t < n_tiles; ++t) {
        const uint8_t* table = comp.data() + lay.off_table + (uint64_t)p12_table_slot(t, d, d_ff) * kP12TableBytes;
        for (int l = 0; l < 64; ++l) {
            uint8_t w[12];
            memcpy(w, comp.data() + lay.off_payload + (uint64_t)t * kP12TileBytes + l * 12, 12);
            for (int j = 0; j < 8; ++j) {
                const uint32_t code = j < 4 ? (w[8 + j] & 15u) : (uint32_t)(w[8 + j - 4] >> 4);
                out[(uint64_t)t * 512 + l * 8 + j] = (uint16_t)(w[j] | ((uint32_t)table[code] << 8));
            }
        }
    }
    return out;
}

int main() {
    const int d = 192, d_ff = 320, E = 5, n_tokens = 41;       // partial gate/up and down groups
    const uint64_t blob_elems = 3ull * d * d_ff, blob_bytes = blob_elems * 2;
    std::vector<std::vector<uint16_t>> wg(E), wu(E), wd(E);
    std::vector<uint16_t> blobs(E * blob_elems);
    for (int e = 0; e < E; ++e) {
        wg[e].resize((size_t)d_ff * d); wu[e].resize((size_t)d_ff * d); wd[e].resize((size_t)d * d_ff);
        for (auto* m : {&wg[e], &wu[e], &wd[e]})
            for (auto& v : *m) v = bf16_of(next_unit() * 0.2f);
        wg[e][7] = 0; wu[e][11] = 0x0001; wd[e][13] = 0x7f80;      // a zero, a denormal, an infinity: table entries like any other
        pack_expert_blob(d, d_ff, wg[e].data(), wu[e].data(), wd[e].data(), blobs.data() + e * blob_elems);
    }
    wd[0][13] = bf16_of(0.01f);                                    // keep the arithmetic checks finite
    pack_expert_blob(d, d_ff, wg[0].data(), wu[0].data(), wd[0].data(), blobs.data());
    // packed layout: spot checks of the documented tile order
    {
        const uint16_t* b = blobs.data() + 1 * blob_elems;
        const int kch = d / 32;
        CHECK(b[0] == wg[1][0]);                                                   // group 0, chunk 0, gate stripe 0, lane 0
        CHECK(b[(uint64_t)(0 * 16 + 8) * 512 + 3 * 8 + 2] == wu[1][(size_t)3 * d + 2]);      // its up stripe 0, lane 3
        CHECK(b[(uint64_t)(1 * 16 + 2) * 512 + 17 * 8] == wg[1][(size_t)(2 * 16 + 1) * d + 32 + 8]);   // chunk 1, stripe 2, lane 17
        const uint16_t* down = b + 2ull * d * d_ff;
        CHECK(down[5 * 8 + 1] == wd[1][(size_t)5 * d_ff + 1]);
        (void)kch;
    }
    // 12-bit form: bit-exact round trip by hand and through the library's inverse; a blob of arbitrary bits is marked raw
    const uint64_t comp_bytes = p12_layout(blob_bytes / 1024).bytes;
    for (int e = 0; e < E; ++e) {
        std::vector<uint8_t> comp(comp_bytes);
        compress_expert_blob(d, d_ff, blobs.data() + e * blob_elems, comp.data());
        const P12Header* h = reinterpret_cast<const P12Header*>(comp.data());
        CHECK(h->magic == kP12Magic && h->raw == 0 && h->n_tiles == blob_bytes / 1024);
        const std::vector<uint16_t> back = decode_p12(comp, blob_bytes, d, d_ff);
        CHECK(memcmp(back.data(), blobs.data() + e * blob_elems, blob_bytes) == 0);
        std::vector<uint16_t> again(blob_elems, 0xAAAA);
        CHECK(decompress_expert_blob(d, d_ff, comp.data(), again.data()));
        CHECK(memcmp(again.data(), blobs.data() + e * blob_elems, blob_bytes) == 0);
    }
    {
        std::vector<uint16_t> noise(blob_elems);
        for (auto& v : noise) v = (uint16_t)next_u32();
        std::vector<uint8_t> comp(comp_bytes);
        compress_expert_blob(d, d_ff, noise.data(), comp.data());
        CHECK(reinterpret_cast<const P12Header*>(comp.data())->raw == 1);
        CHECK(!decompress_expert_blob(d, d_ff, comp.data(), noise.data()));
    }
    // one expert on the calling thread against plain loops
    std::vector<uint16_t> x((size_t)n_tokens * d);
    for (auto& v : x) v = bf16_of(next_unit() * 2.f);
    auto naive = [&](int e, int t, std::vector<float>& y) {
        std::vector<float> a(d_ff);
        for (int i = 0; i < d_ff; ++i) {
            double g = 0, u = 0;
            for (int j = 0; j < d; ++j) {
                g += (double)f32_of(wg[e][(size_t)i * d + j]) * f32_of(x[(size_t)t * d + j]);
                u += (double)f32_of(wu[e][(size_t)i * d + j]) * f32_of(x[(size_t)t * d + j]);
            }
            a[i] = f32_of(bf16_of((float)(g / (1.0 + std::exp(-g)) * u)));
        }
        y.assign(d, 0.f);
        for (int c = 0; c < d; ++c) {
            double s = 0;
            for (int i = 0; i < d_ff; ++i) s += (double)f32_of(wd[e][(size_t)c * d_ff + i]) * a[i];
            y[c] = (float)s;
        }
    };
    {
        std::vector<float> y((size_t)n_tokens * d), ref;
        host_expert_forward(blobs.data(), d, d_ff, x.data(), n_tokens, y.data());
        double worst = 0, scale = 0;
        for (int t = 0; t < n_tokens; t += 8) {
            naive(0, t, ref);
            for (int c = 0; c < d; ++c) { worst = std::fmax(worst, std::fabs(y[(size_t)t * d + c] - ref[c])); scale = std::fmax(scale, std::fabs(ref[c])); }
        }
        CHECK(scale > 0 && worst <= 2e-2 * scale);
    }
    // the pool's miss pass: shuffled list, several threads, twice on the same pool; then a bad entry
    std::vector<tide_miss> miss;
    for (int t = 0; t < n_tokens; ++t)
        for (int r = 0; r < 2; ++r)
            if ((next_u32() & 3) != 0) miss.push_back(tide_miss{t, (int32_t)((t + r * 2) % E), 0.25f + 0.5f * (next_unit() + 0.5f)});
    for (size_t i = miss.size(); i > 1; --i) std::swap(miss[i - 1], miss[next_u32() % i]);
    for (int threads : {1, 4, 7}) {
        HostPool* pool = host_pool_create(threads);
        CHECK(host_pool_threads(pool) == threads);
        for (int rep = 0; rep < 2; ++rep) {
            std::vector<float> rows((size_t)n_tokens * d, -1.f);
            std::vector<int32_t> toks(n_tokens, -1);
            const int n_rows = host_apply_misses(pool, reinterpret_cast<const uint8_t*>(blobs.data()), blob_bytes, d, d_ff, E, x.data(),
                                                 n_tokens, miss.data(), (int)miss.size(), rows.data(), toks.data());
            CHECK(n_rows > 0 && n_rows <= n_tokens);
            for (int r = 0; r < n_rows; r += 5) {
                CHECK(toks[r] >= 0 && toks[r] < n_tokens && (r == 0 || toks[r] > toks[r - 1]));
                std::vector<float> want(d, 0.f), ref;
                for (const tide_miss& m : miss)
                    if (m.token == toks[r]) {
                        naive(m.expert, m.token, ref);
                        for (int c = 0; c < d; ++c) want[c] += m.weight * ref[c];
                    }
                double worst = 0, scale = 0;
                for (int c = 0; c < d; ++c) { worst = std::fmax(worst, std::fabs(rows[(size_t)r * d + c] - want[c])); scale = std::fmax(scale, std::fabs(want[c])); }
                CHECK(scale > 0 && worst <= 2e-2 * scale);
            }
        }
        std::vector<tide_miss> bad = miss;
        bad[bad.size() / 2].expert = E;
        std::vector<float> rows((size_t)n_tokens * d);
        std::vector<int32_t> toks(n_tokens);
        CHECK(host_apply_misses(pool, reinterpret_cast<const uint8_t*>(blobs.data()), blob_bytes, d, d_ff, E, x.data(), n_tokens,
                                bad.data(), (int)bad.size(), rows.data(), toks.data()) == -1);
        host_pool_destroy(pool);
    }
    printf("host sanitize ok\n");
    return 0;
}
