// Lossless 12-bit form of a packed expert blob, used only as the source of refresh copies: the bytes that
// cross the host link shrink to 3/4, the copy kernel rebuilds the bf16 values bit for bit in the cache slot.
//
// A bf16 is sign(1) exponent(8) mantissa(7).  Inside one 16 x 32 tile of trained or Gaussian weights the
// exponents span few binades, so a tile stores one exponent (base: the top of the 16-binade window that holds
// most of its elements) and every element as sign(1) | base - exponent (4) | mantissa(7) = 12 bits.  The rare
// element outside the window (a zero, a denormal, an outlier) goes to a per-expert exception list that is
// applied after the tile decode.  Plain C++: included by the host-side encoder and by the device decoder.
//
//   [0, 64)                    header: magic, n_tiles, n_exceptions, raw (1 = not encoded: copy the raw blob)
//   [64, 64 + pad64(T))        base exponent of each tile, one byte
//   then T x 768 bytes         tile payloads: lane l's 8 elements are 3 dwords at byte 12 l
//   then T x 4 bytes           exception element indices (uint32; capacity T entries)
//   then T x 2 bytes           exception values (bf16 bits)
#pragma once
#include <stdint.h>

namespace tide {

constexpr uint32_t kP12Magic = 0x32315054u;      // "TP12"
constexpr int kP12TileBytes = 768;

struct P12Header {
    uint32_t magic, n_tiles, n_exc, raw;
    uint32_t pad[12];
};
static_assert(sizeof(P12Header) == 64, "header is one 64-byte line");

struct P12Layout {
    uint64_t off_base, off_payload, off_exc_idx, off_exc_val, bytes;
};
constexpr P12Layout p12_layout(uint64_t n_tiles) {        // constexpr: callable from host and device code alike
    P12Layout l{};
    l.off_base = 64;
    l.off_payload = l.off_base + (n_tiles + 63) / 64 * 64;
    l.off_exc_idx = l.off_payload + n_tiles * kP12TileBytes;
    l.off_exc_val = l.off_exc_idx + n_tiles * 4;
    l.bytes = (l.off_exc_val + n_tiles * 2 + 63) / 64 * 64;
    return l;
}

}  // namespace tide
