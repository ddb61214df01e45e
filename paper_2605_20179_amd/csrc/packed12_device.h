// Device-side decoder of the 12-bit blob form (packed12.h): a lane's three dwords and its tile's table -> the
// lane's 16 bytes of bf16, four elements at a time with byte permutes.
#pragma once
#include <hip/hip_runtime.h>

#include "packed12.h"

namespace tide {

struct P12Words {
    uint32_t a0, a1, b;
};

// high bytes of four elements: byte j of `codes` holds a 4-bit table index in its low half
__device__ inline uint32_t p12_high4(uint32_t codes, const uint4& table) {
    const uint32_t sel = codes & 0x07070707u;
    // v_perm_b32(s0, s1, sel): selector 0..3 takes a byte of s1, 4..7 a byte of s0
    const uint32_t lower = __builtin_amdgcn_perm(table.y, table.x, sel);     // entries 0..7
    const uint32_t upper = __builtin_amdgcn_perm(table.w, table.z, sel);     // entries 8..15
    const uint32_t bit3 = codes & 0x08080808u, top = bit3 << 4;
    const uint32_t mask = (top - (bit3 >> 3)) | top;                          // 0xff in the bytes whose index is >= 8
    return (upper & mask) | (lower & ~mask);
}

__device__ inline uint4 p12_decode(const P12Words& w, const uint4& table) {
    const uint32_t h0 = p12_high4(w.b & 0x0f0f0f0fu, table);                  // elements 0..3
    const uint32_t h1 = p12_high4((w.b >> 4) & 0x0f0f0f0fu, table);           // elements 4..7
    uint4 o;                                                                   // element j = low byte | high byte << 8
    o.x = __builtin_amdgcn_perm(h0, w.a0, 0x05010400u);
    o.y = __builtin_amdgcn_perm(h0, w.a0, 0x07030602u);
    o.z = __builtin_amdgcn_perm(h1, w.a1, 0x05010400u);
    o.w = __builtin_amdgcn_perm(h1, w.a1, 0x07030602u);
    return o;
}

}  // namespace tide
