// Device-side decoder of the 12-bit blob form (packed12.h): a lane's three dwords and its tile's table -> the
// lane's 16 bytes of bf16, four elements at a time with byte permutes.
#pragma once
#include <hip/hip_runtime.h>

#include "packed12.h"

namespace tide {

struct P12Words {
    uint32_t a0, a1, b;
};

// high bytes of four elements: the low half of byte j of `codes` holds a 4-bit table index (the high half is ignored)
__device__ inline uint32_t p12_high4(uint32_t codes, const uint4& table) {
    const uint32_t sel = codes & 0x07070707u;
    // v_perm_b32(s0, s1, sel): selector 0..3 takes a byte of s1, 4..7 a byte of s0
    const uint32_t lower = __builtin_amdgcn_perm(table.y, table.x, sel);     // entries 0..7
    const uint32_t upper = __builtin_amdgcn_perm(table.w, table.z, sel);     // entries 8..15
    // byte j of the result: byte j of `upper` where the index is >= 8 (selector j + 4), else byte j of `lower`
    const uint32_t pick = ((codes >> 1) & 0x04040404u) | 0x03020100u;
    return __builtin_amdgcn_perm(upper, lower, pick);
}

__device__ inline uint4 p12_decode(const P12Words& w, const uint4& table) {
    const uint32_t h0 = p12_high4(w.b, table);                                // elements 0..3
    const uint32_t h1 = p12_high4(w.b >> 4, table);                           // elements 4..7
    uint4 o;                                                                   // element j = low byte | high byte << 8
    o.x = __builtin_amdgcn_perm(h0, w.a0, 0x05010400u);
    o.y = __builtin_amdgcn_perm(h0, w.a0, 0x07030602u);
    o.z = __builtin_amdgcn_perm(h1, w.a1, 0x05010400u);
    o.w = __builtin_amdgcn_perm(h1, w.a1, 0x07030602u);
    return o;
}

}  // namespace tide
