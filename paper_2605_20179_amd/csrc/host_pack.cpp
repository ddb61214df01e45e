// Packing of expert weights into the streaming layout and into its lossless 12-bit form (host only).
#include "host_pack.h"

#include <algorithm>
#include <cstring>

#include "host_experts.h"
#include "packed12.h"

namespace tide {

namespace {

constexpr int kGateUpGroup = kHostGateUpGroup, kDownGroup = kHostDownGroup;

// One 16-row x 32-column tile of a row-major matrix -> 512 contiguous elements, lane-major:
// lane l holds row stripe*16 + l%16, columns kc*32 + (l/16)*8 .. +7 (the A operand of the 16x16x32 MFMA).
void pack_tile(const uint16_t* src, int cols, int stripe, int kc, uint16_t* tile) {
    for (int l = 0; l < 64; ++l)
        memcpy(tile + l * 8, src + (int64_t)(stripe * 16 + (l & 15)) * cols + kc * 32 + (l >> 4) * 8, 16);
}

// Streaming order of the tiles.  The 16-row stripes of a matrix are taken in groups -- the stripes one
// workgroup of the GEMM kernels consumes together -- and inside a group the K chunk is the slow index,
// so a workgroup walks one contiguous region front to back (16 KiB per chunk for a full group).
//   gate/up: a group is 8 SwiGLU column blocks = their 8 gate stripes, then their 8 up stripes
//   down:    a group is 16 stripes (256 output columns)
// A last, partial group holds fewer stripes and is laid out the same way.
void pack_gate_up(const uint16_t* wg, const uint16_t* wu, int d_ff, int d, uint16_t* dst) {
    const int kchunks = d / 32, blocks = d_ff / 16;
    for (int g = 0; g * kGateUpGroup < blocks; ++g) {
        const int ng = std::min(kGateUpGroup, blocks - g * kGateUpGroup);
        uint16_t* base = dst + (int64_t)g * 2 * kGateUpGroup * kchunks * 512;
        for (int kc = 0; kc < kchunks; ++kc)
            for (int j = 0; j < ng; ++j) {
                pack_tile(wg, d, g * kGateUpGroup + j, kc, base + ((int64_t)kc * 2 * ng + j) * 512);
                pack_tile(wu, d, g * kGateUpGroup + j, kc, base + ((int64_t)kc * 2 * ng + ng + j) * 512);
            }
    }
}
void pack_down(const uint16_t* wd, int d, int d_ff, uint16_t* dst) {
    const int kchunks = d_ff / 32, stripes = d / 16;
    for (int g = 0; g * kDownGroup < stripes; ++g) {
        const int ng = std::min(kDownGroup, stripes - g * kDownGroup);
        uint16_t* base = dst + (int64_t)g * kDownGroup * kchunks * 512;
        for (int kc = 0; kc < kchunks; ++kc)
            for (int j = 0; j < ng; ++j) pack_tile(wd, d_ff, g * kDownGroup + j, kc, base + ((int64_t)kc * ng + j) * 512);
    }
}

}  // namespace

void pack_expert_blob(int d, int d_ff, const uint16_t* wg, const uint16_t* wu, const uint16_t* wd, uint16_t* blob) {
    pack_gate_up(wg, wu, d_ff, d, blob);
    pack_down(wd, d, d_ff, blob + 2 * (int64_t)d * d_ff);
}

void compress_expert_blob(int d, int d_ff, const uint16_t* src, uint8_t* out) {
    const uint32_t n_tiles = (uint32_t)(3ull * d * d_ff / 512);
    const P12Layout lay = p12_layout(n_tiles);
    memset(out, 0, lay.bytes);
    P12Header* h = reinterpret_cast<P12Header*>(out);
    h->magic = kP12Magic;
    h->n_tiles = n_tiles;
    for (uint32_t t = 0; t < n_tiles; ++t) {
        const uint16_t* tile = src + (uint64_t)t * 512;
        // the tile's table: its distinct high bytes in ascending order
        bool seen[256] = {false};
        for (int i = 0; i < 512; ++i) seen[tile[i] >> 8] = true;
        uint8_t code_of[256];
        uint8_t* table = out + lay.off_table + (uint64_t)p12_table_slot(t, d, d_ff) * kP12TableBytes;
        int n = 0;
        for (int v = 0; v < 256; ++v)
            if (seen[v]) {
                if (n == 16) {                 // a 17th high byte: this blob stays in its bf16 form
                    memset(out + lay.off_payload, 0, lay.bytes - lay.off_payload);
                    h->raw = 1;
                    return;
                }
                code_of[v] = (uint8_t)n;
                table[n++] = (uint8_t)v;
            }
        uint32_t* words = reinterpret_cast<uint32_t*>(out + lay.off_payload + (uint64_t)t * kP12TileBytes);
        for (int l = 0; l < 64; ++l) {
            uint32_t a[2] = {0, 0}, b = 0;
            for (int j = 0; j < 8; ++j) {
                const uint32_t v = tile[l * 8 + j];
                a[j >> 2] |= (v & 0xffu) << (8 * (j & 3));
                b |= (uint32_t)code_of[v >> 8] << (8 * (j & 3) + (j < 4 ? 0 : 4));
            }
            words[l * 3 + 0] = a[0];
            words[l * 3 + 1] = a[1];
            words[l * 3 + 2] = b;
        }
    }
}

bool decompress_expert_blob(int d, int d_ff, const uint8_t* comp, uint16_t* blob) {
    const uint32_t n_tiles = (uint32_t)(3ull * d * d_ff / 512);
    const P12Layout lay = p12_layout(n_tiles);
    const P12Header* h = reinterpret_cast<const P12Header*>(comp);
    if (h->magic != kP12Magic || h->n_tiles != n_tiles || h->raw) return false;
    for (uint32_t t = 0; t < n_tiles; ++t) {
        const uint32_t* words = reinterpret_cast<const uint32_t*>(comp + lay.off_payload + (uint64_t)t * kP12TileBytes);
        const uint8_t* table = comp + lay.off_table + (uint64_t)p12_table_slot(t, d, d_ff) * kP12TableBytes;
        for (int l = 0; l < 64; ++l)
            for (int j = 0; j < 8; ++j)
                blob[(uint64_t)t * 512 + l * 8 + j] = p12_element(words[l * 3], words[l * 3 + 1], words[l * 3 + 2], table, j);
    }
    return true;
}

}  // namespace tide
