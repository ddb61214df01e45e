// Host-side preparation of expert weights: the packed streaming layout of a blob and its lossless 12-bit
// form.  Plain C++ with no HIP in it, so that it can also be built and run under the host sanitizers.
#pragma once
#include <stdint.h>

namespace tide {

// wg / wu [d_ff][d], wd [d][d_ff] row-major bf16 -> blob (3 * d * d_ff elements) in the layout tide_pack_expert documents.
void pack_expert_blob(int d, int d_ff, const uint16_t* wg, const uint16_t* wu, const uint16_t* wd, uint16_t* blob);

// packed blob of an expert with hidden size d and intermediate size d_ff -> its 12-bit form (packed12.h),
// p12_layout(3 * d * d_ff / 512).bytes long.
void compress_expert_blob(int d, int d_ff, const uint16_t* src, uint8_t* out);

// the inverse: false (blob untouched) when `comp` is not a compressed blob of that shape or is marked raw
bool decompress_expert_blob(int d, int d_ff, const uint8_t* comp, uint16_t* blob);

}  // namespace tide
