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

void compress_expert_blob(uint64_t blob_bytes, const uint16_t* src, uint8_t* out) {
    const uint32_t n_tiles = (uint32_t)(blob_bytes / 1024);
    const P12Layout lay = p12_layout(n_tiles);
    memset(out, 0, lay.bytes);
    P12Header* h = reinterpret_cast<P12Header*>(out);
    h->magic = kP12Magic;
    h->n_tiles = n_tiles;
    uint32_t* exc_idx = reinterpret_cast<uint32_t*>(out + lay.off_exc_idx);
    uint16_t* exc_val = reinterpret_cast<uint16_t*>(out + lay.off_exc_val);
    uint32_t n_exc = 0;
    for (uint32_t t = 0; t < n_tiles && !h->raw; ++t) {
        const uint16_t* tile = src + (uint64_t)t * 512;
        // base: the top of the 16-binade window that holds the most elements of the tile (the highest such window)
        uint32_t hist[256 + 16] = {0};
        for (int i = 0; i < 512; ++i) hist[(tile[i] >> 7) & 0xff]++;
        uint32_t base = 15, in_window = 0, best = 0;
        for (uint32_t e = 0; e < 16; ++e) in_window += hist[e];
        best = in_window;
        for (uint32_t top = 16; top < 256; ++top) {
            in_window += hist[top] - hist[top - 16];
            if (in_window >= best) { best = in_window; base = top; }
        }
        out[lay.off_base + t] = (uint8_t)base;
        uint32_t* words = reinterpret_cast<uint32_t*>(out + lay.off_payload + (uint64_t)t * kP12TileBytes);
        for (int l = 0; l < 64; ++l) {
            uint32_t code[8];
            for (int j = 0; j < 8; ++j) {
                const uint32_t v = tile[l * 8 + j], e = (v >> 7) & 0xff;
                uint32_t delta = base - e;             // wraps for an exponent above the window
                if (delta > 15) {                      // outside the tile's 16-binade window: listed
                    if (n_exc == n_tiles) { h->raw = 1; break; }
                    exc_idx[n_exc] = t * 512 + l * 8 + j;
                    exc_val[n_exc++] = (uint16_t)v;
                    delta = 15;
                }
                code[j] = ((v >> 15) << 11) | (delta << 7) | (v & 0x7f);
            }
            if (h->raw) break;
            words[l * 3 + 0] = code[0] | (code[1] << 12) | ((code[2] & 0xff) << 24);
            words[l * 3 + 1] = (code[2] >> 8) | (code[3] << 4) | (code[4] << 16) | ((code[5] & 0xf) << 28);
            words[l * 3 + 2] = (code[5] >> 4) | (code[6] << 8) | (code[7] << 20);
        }
    }
    h->n_exc = h->raw ? 0 : n_exc;
}



}  // namespace tide
