// Lossless 12-bit form of a packed expert blob: 3/4 of the bytes (plus 16 per tile), every bf16 rebuilt bit for
// bit.  It is what crosses the host link in a refresh copy and, when the context keeps its cache slots in this
// form, what the expert GEMMs stream from HBM and decode in registers.
//
// A bf16 is sign(1) exponent(8) mantissa(7): its low byte is the exponent's last bit and the mantissa, its high
// byte the sign and the upper seven exponent bits.  Inside one 16 x 32 tile of trained or Gaussian weights the
// low bytes look random, but the high bytes take few distinct values (both signs of five to seven pairs of
// binades).  A tile therefore stores the low byte of every element as it is, a table of up to 16 high bytes, and
// per element a 4-bit index into that table.  A tile with more than 16 distinct high bytes cannot be encoded:
// the whole blob is then marked raw and used in its bf16 form (Gaussian weights: a few tiles in a million).
//
//   [0, 128)                   header: magic, n_tiles, raw (1 = not encoded: use the bf16 blob); one 128-byte cache
//                              line, so that every 768-byte payload below is six whole lines
//   [128, 128 + 768 T)         tile payloads in tile order.  Lane l (the 8 consecutive elements 8l .. 8l+7 of the
//                              tile) owns the 3 dwords at byte 12 l:
//                                a0: low bytes of elements 0..3          a1: low bytes of elements 4..7
//                                b : byte j = index of element j | index of element 4+j << 4
//   then 16 T bytes            tables: 16 high bytes per tile, unused entries zero.  Inside a stripe group of the packed
//                              layout the payloads are ordered K chunk first, the tables stripe first (table of stripe
//                              j, chunk c of a group at the group's first tile + j * chunks + c): a wave of the expert
//                              GEMMs walks the chunks of its own stripes, so the tables it needs next are contiguous
//
// Plain C++: included by the host-side encoder / decoder and by the device code.
#pragma once
#include <stdint.h>

namespace tide {

constexpr uint32_t kP12Magic = 0x32315054u;      // "TP12"
constexpr int kP12TileBytes = 768;
constexpr int kP12TableBytes = 16;
constexpr int kP12HeaderBytes = 128;

struct P12Header {
    uint32_t magic, n_tiles, raw;
    uint32_t pad[29];
};
static_assert(sizeof(P12Header) == kP12HeaderBytes, "header is one 128-byte line");

struct P12Layout {
    uint64_t off_payload, off_table, bytes;
};
constexpr P12Layout p12_layout(uint64_t n_tiles) {        // constexpr: callable from host and device code alike
    P12Layout l{};
    l.off_payload = kP12HeaderBytes;
    l.off_table = l.off_payload + n_tiles * kP12TileBytes;                  // 768 = 6 x 128: still 128-byte aligned
    l.bytes = (l.off_table + n_tiles * kP12TableBytes + 63) / 64 * 64;
    return l;
}

// Where the table of payload tile `tile` sits (in tables from the start of the table region), for a blob of an expert
// with hidden size d and intermediate size d_ff: the packed layout's groups (8 SwiGLU column blocks = up to 16 gate and
// up stripes; then 16 down stripes), a last group with fewer stripes included.
constexpr uint32_t p12_table_slot(uint32_t tile, int d, int d_ff) {
    const uint32_t kcd = d / 32, blocks = d_ff / 16, kci = d_ff / 32, stripes = d / 16, gate_up = 2 * blocks * kcd;
    if (tile < gate_up) {
        const uint32_t span = 2 * 8 * kcd, g = tile / span, base = g * span;
        const uint32_t width = 2 * (blocks - 8 * g < 8 ? blocks - 8 * g : 8);
        return base + ((tile - base) % width) * kcd + (tile - base) / width;
    }
    const uint32_t t = tile - gate_up, span = 16 * kci, g = t / span, base = g * span;
    const uint32_t width = stripes - 16 * g < 16 ? stripes - 16 * g : 16;
    return gate_up + base + ((t - base) % width) * kci + (t - base) / width;
}

// element j (0..7) of a lane from the lane's three dwords and the tile's table
inline uint16_t p12_element(uint32_t a0, uint32_t a1, uint32_t b, const uint8_t* table, int j) {
    const uint32_t low = ((j < 4 ? a0 : a1) >> (8 * (j & 3))) & 0xffu;
    const uint32_t code = (b >> (8 * (j & 3) + (j < 4 ? 0 : 4))) & 0xfu;
    return (uint16_t)(low | ((uint32_t)table[code] << 8));
}

}  // namespace tide
