// Host-core execution of missed experts (Sec. 3.3: tokens routed to an expert that is not
// resident are evaluated by CPU experts while the GPU evaluates the hits).  Plain C++,
// no HIP: worker threads read the packed expert blobs in place from host memory.
#pragma once
#include <stdint.h>

#include "tide.h"

namespace tide {

// the packed layout's group sizes (tide_pack_expert); tide_api.hip checks them against the kernels' constants
constexpr int kHostGateUpGroup = 8;
constexpr int kHostDownGroup = 16;

struct HostPool;
// n_threads >= 1 threads work on a call, the calling thread included
HostPool* host_pool_create(int n_threads);
void host_pool_destroy(HostPool* p);
int host_pool_threads(const HostPool* p);

// y[t][:] = e(x_t) for m token states (bf16 [m][d]) through one packed blob, on the calling thread.
void host_expert_forward(const void* blob, int d, int d_ff, const uint16_t* x, int m, float* y);

// Sums a miss list into rows: for every token with at least one listed miss
//   y_rows[r][:] = sum over the token's misses, in list order, of weight * e_expert(x_token)
// tokens_out[r] is the token of row r (ascending).  Returns the number of rows, or -1 when an entry
// names a token outside [0, n_tokens) or an expert outside [0, n_experts).
//   blobs + e * stride  packed blob of expert e (host memory)
//   x                   bf16 [n_tokens][d] (host)
//   y_rows              fp32 [min(n, n_tokens)][d] at least; tokens_out int32 [same]
//   skip_expert         [n_experts] bytes or null: entries of experts with a non-zero byte are left out (someone
//                       else evaluates them)
int host_apply_misses(HostPool* pool, const uint8_t* blobs, uint64_t stride, int d, int d_ff, int n_experts,
                      const uint16_t* x, int n_tokens, const tide_miss* miss, int n, float* y_rows,
                      int32_t* tokens_out, const uint8_t* skip_expert = nullptr);

}  // namespace tide
