/*
 * libtide -- the per-denoise-step MoE expert layer of TIDE against a
 * GPU-resident expert cache, the interval hit counter, and the top-B refresh
 * with its host-to-device copy plan, for one AMD MI355X (gfx950).
 *
 * Paper vocabulary used below (Sec. 3.1, Sec. 3.3, Alg. 1):
 *   E        routed experts per layer            k   experts per token
 *   B        GPU expert budget (here: capacity)  tau refresh interval
 *   H        hit counter: tokens each expert processed since the last refresh
 *   E^GPU    resident set, E^CPU the rest (held by the caller in pinned host memory)
 *
 * Conventions
 *   - Every entry point returns 0 (TIDE_OK) or a negative TIDE_E_* code;
 *     tide_last_error() returns a text for the last failure on that context.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  The library never frees caller memory and never keeps a
 *     caller pointer beyond the call unless stated (registered expert blobs).
 *   - bf16 = upper 16 bits of an IEEE fp32, carried as uint16_t.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls on one context must be issued in stream order on ONE stream: the
 *     context owns a single workspace shared by all of its layers (the layers of a
 *     stack that do not depend on each other go through tide_moe_stack_step, which
 *     overlaps them on streams and workspaces of its own).
 *   - Nothing is computed on the CPU: if no gfx950 device is usable,
 *     tide_create fails with TIDE_E_HIP.
 */
#ifndef TIDE_H_
#define TIDE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIDE_OK          0
#define TIDE_E_INVAL    (-1)   /* null pointer, bad enum, bad layer index, size not supported   */
#define TIDE_E_RANGE    (-2)   /* capacity / token count / expert id outside what ctx was built for */
#define TIDE_E_STATE    (-3)   /* call order: experts not registered, placement not set, ...     */
#define TIDE_E_HIP      (-4)   /* a HIP runtime call failed; text in tide_last_error             */
#define TIDE_E_NOMEM    (-5)

#define TIDE_GATING_SOFTMAX 0  /* softmax over E, weights renormalised over the k selected */
#define TIDE_GATING_SIGMOID 1  /* sigmoid per expert, weights renormalised over the k selected */
#define TIDE_BIAS_NONE   0
#define TIDE_BIAS_LOGIT  1     /* bias added to the router logit before the gate */
#define TIDE_BIAS_SELECT 2     /* bias added to the gate score for selection only, not to the weights */
#define TIDE_RESIDENT_BF16 0   /* a cache slot holds the expert's packed bf16 blob */
#define TIDE_RESIDENT_P12  1   /* a cache slot holds the blob's lossless 12-bit form (tide_compress_expert) */

typedef struct tide_ctx tide_ctx;

/* One token routed to an expert that is not resident ("miss", Alg. 1 token routing). */
typedef struct { int32_t token; int32_t expert; float weight; } tide_miss;

/* One host-to-device expert copy of a refresh (Alg. 1 refresh step). */
typedef struct { int32_t expert; int32_t slot; uint64_t host_offset; uint64_t bytes; } tide_copy;

typedef struct {
    int32_t d;           /* hidden size; multiple of 64                                  */
    int32_t n_experts;   /* E, 1..512                                                    */
    int32_t top_k;       /* k, 1..min(E,16)                                              */
    int32_t d_ff;        /* SwiGLU intermediate size I; multiple of 64                   */
    int32_t n_shared;    /* 0 or 1 always-resident shared expert (weight 1, not counted) */
    int32_t n_layers;    /* independent MoE layers, each with its own cache and counter  */
    int32_t capacity;    /* cache slots per layer (the paper's B), 1..E                  */
    int32_t max_tokens;  /* largest n_tokens a step may carry, 1..65535                  */
    int32_t gating;      /* TIDE_GATING_*                                                */
    int32_t bias_mode;   /* TIDE_BIAS_*                                                  */
    int32_t resident_format; /* TIDE_RESIDENT_*: the form a cache slot keeps its blob in  */
} tide_config;

/* ---- set-up --------------------------------------------------------------------- */

/* Allocates the context on the current HIP device: per layer `capacity` weight slots
 * (one packed bf16 blob each, whatever resident_format says they will hold),
 * the hit counter H[E] (zero), the placement tables (all slots empty), and one
 * workspace sized by max_tokens.  Creates two streams of default priority: one for
 * refresh copies, one on which a step's large work items run beside the small ones.
 * resident_format: TIDE_RESIDENT_BF16 (0; a zeroed field means this) or TIDE_RESIDENT_P12,
 * both described with tide_register_compressed below. */
int tide_create(const tide_config* cfg, tide_ctx** out);
int tide_destroy(tide_ctx* ctx);
/* Text of the last error on ctx (ctx == NULL: last error of a failed tide_create). */
const char* tide_last_error(const tide_ctx* ctx);

/* Bytes of one packed expert blob: 3 * d * d_ff * 2. */
uint64_t tide_expert_blob_bytes(const tide_config* cfg);

/* Host-side packing of one expert e(x) = Wd (silu(Wg x) * (Wu x)) (Alg. 1, "output = e(x)")
 * from row-major bf16 matrices wg[d_ff][d], wu[d_ff][d], wd[d][d_ff] (host) into the
 * library's streaming layout at blob_host (host, tide_expert_blob_bytes bytes).
 * The blob is what lives in pinned host memory and in a cache slot, byte for byte.
 * Layout: 16-row x 32-column tiles of 512 elements, lane-major (lane l: row l%16 of the
 * tile, columns (l/16)*8..+7).  First the gate and up matrices interleaved: groups of 8
 * SwiGLU column blocks (16 rows of Wg and of Wu each); inside a group, for each K chunk
 * of 32 columns, the group's gate tiles then its up tiles.  Then the down matrix: groups
 * of 16 row stripes; inside a group, for each K chunk, the group's tiles.  A last group
 * with fewer blocks or stripes is laid out the same way. */
int tide_pack_expert(const tide_config* cfg, const uint16_t* wg_host, const uint16_t* wu_host,
                     const uint16_t* wd_host, void* blob_host);

/* Registers the host master copy of a layer's E packed blobs: expert e starts at
 * host_blobs + e * blob_stride.  The memory must be pinned (hipHostMalloc / torch
 * pin_memory) and stay valid and unchanged until tide_destroy: the refresh's copy kernel
 * and the miss pass read it in place from the GPU, asynchronously.  Pageable memory is
 * refused with TIDE_E_INVAL.  Borrowed, never written, never freed. */
int tide_register_experts(tide_ctx* ctx, int layer, const void* host_blobs, uint64_t blob_stride);

/* A lossless 12-bit form of the packed blobs: about 3/4 of the bytes, every weight rebuilt bit for bit.
 * Format, per 16 x 32 tile: the low byte of every bf16 as it is (last exponent bit and mantissa), a table of
 * the tile's distinct high bytes (sign and upper exponent bits; at most 16), and a 4-bit table index per
 * element: 768 + 16 bytes instead of 1024.  A blob with a tile of more than 16 distinct high bytes (a few
 * tiles in a million for Gaussian weights) is marked "raw" and used in its bf16 form everywhere.
 * Two uses, both needing the raw blobs registered as well (the miss paths read those):
 *   - resident_format == TIDE_RESIDENT_BF16: optional SOURCE OF REFRESH COPIES, so that 3/4 of the bytes
 *     cross the host link; the copy kernel rebuilds the bf16 blob in the cache slot (or staging blob).
 *   - resident_format == TIDE_RESIDENT_P12: required; the cache slots keep the compressed blob as it is
 *     (tide_set_resident, tide_set_shared, every refresh copy and tide_read_slot then move compressed
 *     blobs) and the expert GEMMs decode it in registers: the same outputs bit for bit from 3/4 of the
 *     HBM bytes.  It pays where a step is bound by the weight bytes (small token counts); a large work
 *     item then holds at most 192 rows instead of 256.  The shared expert's slot keeps the 12-bit form
 *     only when max_tokens <= 64: it sees every token of a step, and work items of more than four
 *     16-token tiles run faster from the bf16 blob (tide_read_slot returns whichever form the slot holds).
 *   tide_compressed_blob_bytes  size of one compressed blob (a multiple of 64)
 *   tide_compress_expert        host: packed blob (tide_pack_expert) -> compressed blob
 *   tide_decompress_expert      host: the inverse; TIDE_E_INVAL for a blob marked raw or of another configuration
 *   tide_register_compressed    expert e at comp_host_blobs + e * comp_stride; pinned host memory, 64-byte
 *                               aligned, valid and unchanged until tide_destroy; NULL goes back to raw copies
 *                               (bf16 slots only).  Synchronises the device.  TIDE_E_INVAL for pageable memory
 *                               or a blob that is not of this configuration, TIDE_E_STATE before
 *                               tide_register_experts.  With 12-bit slots the call also withdraws the layer's
 *                               placement (the slots were filled from the blobs registered before): call
 *                               tide_set_resident again before the next step or refresh. */
uint64_t tide_compressed_blob_bytes(const tide_config* cfg);
int tide_compress_expert(const tide_config* cfg, const void* blob_host, void* comp_host);
int tide_decompress_expert(const tide_config* cfg, const void* comp_host, void* blob_host);
int tide_register_compressed(tide_ctx* ctx, int layer, const void* comp_host_blobs, uint64_t comp_stride);

/* Copies one packed blob (host) into the layer's always-resident shared-expert slot.
 * Synchronous.  Required before the first step when n_shared == 1. */
int tide_set_shared(tide_ctx* ctx, int layer, const void* blob_host);

/* Initial placement (the cold start E^GPU): expert experts_host[s] goes to slot s for
 * s < n (n <= capacity; -1 leaves a slot empty; remaining slots are emptied).
 * Copies from the registered host blobs, synchronous.  Does not touch H. */
int tide_set_resident(tide_ctx* ctx, int layer, const int32_t* experts_host, int n);

/* ---- the per-step hot path -------------------------------------------------------- */

/* One MoE layer at one denoise step over n_tokens tokens (Alg. 1, token routing):
 *   router logits z = X W_r^T (fp32), gate, top-k, routing weights renormalised over
 *   the k selected; H[e] += tokens routed to e (all experts, resident or not);
 *   out[n] = shared(x_n) + sum over the token's selected experts that are RESIDENT of
 *            w * e(x_n)                      (bf16 operands, fp32 accumulation);
 *   every selected expert that is not resident is appended to the miss list as
 *   (token, expert, weight), ordered by token then by rank in the token's top-k list.
 * Adding sum over the miss list of weight * e(x_token) to out reproduces the full MoE
 * output: placement never changes what is computed (Sec. 3.3 "Lossless Inference").
 *
 *   hidden_dev      bf16 [n_tokens][d] row-major                               (in)
 *   router_w_dev    fp32 [E][d] row-major                                      (in)
 *   router_bias_dev fp32 [E], or NULL when bias_mode == TIDE_BIAS_NONE         (in)
 *   out_dev         fp32 [n_tokens][d]                                         (out)
 *   miss_dev        tide_miss[miss_cap], n_miss_dev int32[1]                   (out)
 *                   *n_miss_dev is always the full number of misses; only the first
 *                   miss_cap entries are written (miss_cap >= n_tokens*k never truncates)
 *   topk_idx_dev    int32 [n_tokens][k], topk_w_dev fp32 [n_tokens][k]; may be NULL (out)
 * Asynchronous on hip_stream.  If a refresh issued copies for this layer, the expert
 * GEMMs of this call wait for them on the device; routing does not.
 * n_tokens == 0 is allowed (writes *n_miss_dev = 0). */
int tide_moe_step(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens,
                  const float* router_w_dev, const float* router_bias_dev,
                  float* out_dev, tide_miss* miss_dev, int miss_cap, int32_t* n_miss_dev,
                  int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream);

/* tide_moe_step for callers that cannot allocate device memory or let a library do it on their behalf -- code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * (bit for bit) and same errors as tide_moe_step; the difference is where the step's workspace lives (partial
 * router logits, routing tables, slot-sorted row lists, work items, SwiGLU activations, per-row expert outputs):
 * not in the context's own allocation but in ONE array of TIDE_NOALLOC_SCRATCH_BYTES bytes that the library
 * holds in each GPU's memory from load until the process ends.  The call performs no hipMalloc / hipFree and
 * calls no allocating routine.
 *   - A step whose workspace does not fit is refused with TIDE_E_RANGE and nothing is queued (the need grows with
 *     n_tokens * (top_k + n_shared) * (4 d + 2 d_ff) bytes: 32 MiB hold e.g. 320 tokens at d = 2048, d_ff = 512,
 *     top-8 + shared, or 192 tokens at d = 4096, d_ff = 1024).
 *   - TIDE_E_STATE while tide_profile is on (event-stamped launches create events).
 *   - Every context on a GPU shares that GPU's array and the array keeps the last call's contents; nothing in it has
 *     to start at zero.  Calls that overlap in time on one GPU (two streams, two contexts, two threads) race: issue
 *     them in stream order on one stream, like the other calls of a context.
 *   - The step histogram (tide_step_histogram) and the running totals (tide_counters) stay with the context. */
#define TIDE_NOALLOC_SCRATCH_BYTES (32u << 20)
int tide_moe_step_noalloc(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens,
                          const float* router_w_dev, const float* router_bias_dev,
                          float* out_dev, tide_miss* miss_dev, int miss_cap, int32_t* n_miss_dev,
                          int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream);
/* TIDE_NOALLOC_SCRATCH_BYTES as the loaded library was built with. */
uint64_t tide_noalloc_scratch_bytes(void);

/* One denoise step of a STACK of independent MoE layers (layers first_layer .. first_layer + n_layers - 1, each with
 * its own router, hidden states, cache, counter and output): the same results, bit for bit, as tide_moe_step called
 * for each layer in turn -- but the call states that the layers do not depend on each other within the step (no
 * layer's input is another's output), so the library runs consecutive layers on two internal streams with a
 * workspace each: one layer's routing, split and combine run beside the other's expert GEMMs, and the tail of one
 * layer's GEMM launches is filled by the next layer's.  Everything is ordered behind the work already queued on
 * hip_stream, and work queued on hip_stream afterwards runs behind all layers.
 *   hidden_dev, router_w_dev, router_bias_dev, out_dev, miss_dev, n_miss_dev: HOST arrays of n_layers device
 *   pointers, entry i for layer first_layer + i, each as tide_moe_step takes it (router_bias_dev may be NULL when
 *   bias_mode == TIDE_BIAS_NONE; miss_dev may be NULL when miss_cap == 0); the arrays are read before the call returns.
 * The lanes (two workspaces of the context's size, four streams) are allocated by the first call.  TIDE_E_STATE
 * while host workers are active.  tide_step_histogram / tide_read_work_items afterwards describe the last layer. */
int tide_moe_stack_step(tide_ctx* ctx, int first_layer, int n_layers, const void* const* hidden_dev, int n_tokens,
                        const float* const* router_w_dev, const float* const* router_bias_dev, float* const* out_dev,
                        tide_miss* const* miss_dev, int miss_cap, int32_t* const* n_miss_dev, void* hip_stream);

/* The same step for token states that already carry their expert selections
 * (Alg. 1 takes X = {(x, E_x)} as given): topk_idx_dev / topk_w_dev are INPUTS
 * (expert ids in [0,E), distinct per token; topk_idx_dev 16-byte aligned).  Counts, split, expert evaluation,
 * combine and miss list exactly as tide_moe_step.  An id outside [0,E) is reported as a miss and not counted.
 * A token that names an expert more than once gets the sum the definition gives (each listed pair is evaluated
 * with its own weight) and H counts pairs, not tokens, for it. */
int tide_moe_step_routed(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens,
                         const int32_t* topk_idx_dev, const float* topk_w_dev,
                         float* out_dev, tide_miss* miss_dev, int miss_cap, int32_t* n_miss_dev,
                         void* hip_stream);

/* Evaluates a step's misses on the GPU and adds them to out_dev, which then holds the FULL MoE
 * output: out[token] += weight * e_expert(x_token) for every listed miss, in list order.  The
 * missed experts are not copied into the cache and the placement does not change: the expert
 * GEMMs read the weights in place from the registered pinned host blobs across the host link
 * (Sec. 3.3 sends such tokens to CPU experts instead; the result is the same by the lossless
 * property, the cost is one pass over each missed expert's weights at host-link speed).
 *   hidden_dev  the step's input, as passed to tide_moe_step                      (in)
 *   miss_dev / miss_cap / n_miss_dev  the list that step returned; min(*n_miss_dev, miss_cap)
 *               entries are used; an entry that names an expert outside [0,E) or a token
 *               outside [0,n_tokens) is skipped                                    (in)
 *   out_dev     fp32 [n_tokens][d], the step's resident-partial output             (in/out)
 * Asynchronous on hip_stream; must follow the step on the same stream (it reuses the context's
 * workspace).  Does not touch H or the tables. */
int tide_moe_apply_misses(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens,
                          const tide_miss* miss_dev, int miss_cap, const int32_t* n_miss_dev,
                          float* out_dev, void* hip_stream);

/* Host-core execution of misses (Sec. 3.3, Alg. 1: a token whose expert is not in the GPU set is
 * evaluated by the CPU copy of that expert while the GPU evaluates the hits; the partial results
 * are brought together at the end of the layer).
 *
 * tide_host_experts starts n_threads worker threads (the calling thread of a later
 * tide_moe_apply_misses_host counts as one of them) and allocates the pinned exchange buffers
 * (miss list, token states, result rows, sized by max_tokens); n_threads == 0 stops the workers.
 * Synchronises the device.  While workers exist, every step also queues, on its second stream and
 * right behind its hit/miss split, a small kernel that writes the miss list and the token states it
 * names to those pinned buffers. */
int tide_host_experts(tide_ctx* ctx, int n_threads);

/* Same contract and arguments as tide_moe_apply_misses, but the listed misses are evaluated by the
 * host workers from the registered host blobs (fp32 arithmetic on the bf16 weights and token
 * states), and the per-token sums are added to out_dev by a kernel queued on hip_stream.
 * The call blocks the calling thread until the host work is done; it does NOT wait for the GPU
 * work queued on hip_stream: when hidden_dev / n_tokens / miss_dev / miss_cap / hip_stream are those
 * of the last step issued (and the buffers are untouched since), the list and the token states are
 * the ones that step handed over right after its hit/miss split, so the host cores work while the
 * GPU runs the step's expert GEMMs (layer time = the longer of the two, Sec. 3.3); with other
 * buffers the hand-over is queued now and waits for everything queued on hip_stream.
 * Errors: TIDE_E_STATE without workers or registered experts; TIDE_E_INVAL for a list entry
 * that names a token or an expert out of range (nothing is added then). */
int tide_moe_apply_misses_host(tide_ctx* ctx, int layer, const void* hidden_dev, int n_tokens,
                               const tide_miss* miss_dev, int miss_cap, const int32_t* n_miss_dev,
                               float* out_dev, void* hip_stream);

/* Splits the work of tide_moe_apply_misses_host between the two places a missed expert's weights can be
 * read from: `percent` (0..100, default 0 = Sec. 3.3's design, everything on the host cores) of the
 * step's distinct missed experts, those with the most tokens first, are evaluated by the GPU, which
 * reads their blobs in place over the host link (as tide_moe_apply_misses does) behind the step on
 * hip_stream, while the host workers evaluate the others from host memory.  The sum is the same. */
int tide_host_link_share(tide_ctx* ctx, int percent);

/* Host wall-clock milliseconds of the last tide_moe_apply_misses_host: ms3_host[0] waiting for the
 * list and the token states, [1] the host experts, [2] the whole call. */
int tide_host_miss_ms(tide_ctx* ctx, float* ms3_host);

/* The host workers' whole miss path with host buffers only, no GPU involved: for every listed miss
 * out_host[token][:] += weight * e_expert(x_token), evaluated by n_threads threads (started and
 * stopped inside the call) from packed blobs at blobs_host + expert * blob_stride.
 *   x_host bf16 [n_tokens][d]; miss_host tide_miss[n_miss] in any order; out_host fp32 [n_tokens][d]
 * (in/out).  TIDE_E_INVAL for an entry that names a token or an expert out of range (nothing is added).
 * What tide_moe_apply_misses_host runs between its two kernels, exposed for checking it without a device. */
int tide_host_misses(const tide_config* cfg, const void* blobs_host, uint64_t blob_stride,
                     const uint16_t* x_host, int n_tokens, const tide_miss* miss_host, int n_miss,
                     int n_threads, float* out_host);

/* One expert on the calling host thread, no GPU involved: y_host[t][:] = e(x_t) for m token
 * states x_host (bf16 [m][d], host) through one packed blob (host); y_host fp32 [m][d].
 * The arithmetic of the host workers, exposed for checking it without a device. */
int tide_host_expert(const tide_config* cfg, const void* blob_host, const uint16_t* x_host, int m,
                     float* y_host);

/* ---- interval statistics and refresh ---------------------------------------------- */

/* Copies the layer's hit counter H[E] (tokens per expert since the last reset; Fig. 1
 * caption, Sec. 3.3 "global hit counter") to counts_host after all work queued on
 * hip_stream; reset != 0 zeroes it afterwards.  Synchronises hip_stream. */
int tide_interval_stats(tide_ctx* ctx, int layer, int32_t* counts_host, int reset, void* hip_stream);

/* Overwrites the layer's hit counter H[E] with counts_host (all >= 0), after all work queued on hip_stream:
 * the counterpart of tide_interval_stats, so that a caller can snapshot (H, placement) and replay from it,
 * or carry a counter over from another run.  Synchronises hip_stream. */
int tide_set_counts(tide_ctx* ctx, int layer, const int32_t* counts_host, void* hip_stream);

/* Refresh step (Alg. 1; Sec. 3.3: the GPU set becomes the current top-B by hits).
 * Experts are ranked by (hits descending, currently resident first, lower id first);
 * the first `capacity` form the new resident set.  Leaving experts, ordered by
 * (hits ascending, id), free their slots; entering experts, ordered by (hits descending,
 * id), take the freed slots in that order and then empty slots in ascending order.
 * The entering experts' blobs are copied from the registered host blobs by one kernel on
 * the context's side stream (it reads pinned host memory in place); eviction moves no bytes.  The tables change at once; the next
 * step's expert GEMMs wait for the copies.
 *   counts_host     int32 [E] to rank by, or NULL = the layer's own H               (in)
 *   capacity        size of the new resident set, 0..ctx capacity                   (in)
 *   reset_counts    != 0: zero H afterwards (per-interval counting)                 (in)
 *   resident_out    int32 [ctx capacity]: expert in each slot after the refresh, -1 = empty (host, out, may be NULL)
 *   plan_out        tide_copy [ctx capacity] (host, out, may be NULL), *n_copies_out entries
 * Synchronises hip_stream (the plan is needed on the host to queue the copies). */
int tide_refresh(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts,
                 int32_t* resident_out, tide_copy* plan_out, int* n_copies_out, void* hip_stream);

/* The same refresh without the host round trip: selection, plan, counter reset and copies are queued and the call
 * returns at once.  Nothing on the host needs the plan to queue the copies -- the copy kernel reads the plan, and
 * how many copies it holds, from the pinned block the selection kernel writes -- so hip_stream is NOT synchronised;
 * the side stream waits (on the device) for the selection, i.e. for every earlier step queued on hip_stream.
 * The placement, the tables, the next step's wait for the copies: as tide_refresh.  counts_host, if given, must
 * stay valid until the call returns.  The new resident set and the plan are read later with tide_refresh_result. */
int tide_refresh_async(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts,
                       void* hip_stream);
/* resident_out / plan_out / n_copies_out of the layer's last refresh (any of the three forms), as tide_refresh
 * returns them; after tide_refresh_async it first waits for that refresh's selection kernel.  Valid until the
 * layer's next refresh.  TIDE_E_STATE if the layer has not been refreshed. */
int tide_refresh_result(tide_ctx* ctx, int layer, int32_t* resident_out, tide_copy* plan_out, int* n_copies_out);

/* The same refresh with its effect deferred, so that the host-link copies overlap with the steps that
 * follow instead of holding up the next one: the selection, the plan, the counter reset and the copies are
 * as above, but the newcomers land in staging blobs owned by the layer (allocated on first use: `ctx
 * capacity` blobs) and the layer keeps serving from the OLD placement -- tide_moe_step, tide_get_table and
 * the miss lists see no change -- until tide_commit.  resident_out / plan_out describe the placement that
 * the commit will install.  Until then tide_refresh and tide_refresh_deferred on the layer return
 * TIDE_E_STATE; tide_set_resident cancels the pending refresh. */
int tide_refresh_deferred(tide_ctx* ctx, int layer, const int32_t* counts_host, int capacity, int reset_counts,
                          int32_t* resident_out, tide_copy* plan_out, int* n_copies_out, void* hip_stream);
/* Installs the placement of the pending deferred refresh: hip_stream waits for the staged copies, then (in
 * stream order, i.e. after every step already queued) the staged blobs move into their slots inside HBM and
 * the tables are swapped.  Does not synchronise.  TIDE_E_STATE if nothing is pending. */
int tide_commit(tide_ctx* ctx, int layer, void* hip_stream);

/* Blocks until every refresh copy queued so far for the layer has landed. */
int tide_wait_refresh(tide_ctx* ctx, int layer);
/* The same wait queued on hip_stream instead of blocking the host: work queued on hip_stream afterwards runs
 * once the layer's refresh copies have landed.  A step issued eagerly needs neither call -- it queues this wait
 * ahead of its expert GEMMs itself.  A step REPLAYED from a captured HIP graph does not: the wait is decided
 * when the step is issued, and a graph captured on a settled placement holds none.  After tide_refresh /
 * tide_refresh_async, call tide_wait_refresh, or tide_queue_refresh_wait on the replay's stream, before
 * replaying a captured step of that layer, or the replay may read slots the copies are still writing. */
int tide_queue_refresh_wait(tide_ctx* ctx, int layer, void* hip_stream);

/* Who moves a refresh's expert blobs across the host link (Alg. 1's asynchronous migration), for every later
 * refresh on the context:
 *   TIDE_COPY_KERNEL  one kernel on the side stream that reads pinned host memory in place (default; the only
 *                     engine that can decode the 12-bit form of tide_register_compressed into bf16 slots, and the
 *                     only one tide_refresh_async can use, because the host never sees that call's plan);
 *   TIDE_COPY_DMA     one hipMemcpyAsync per entering expert on the side stream, of the bytes the slot keeps
 *                     (the bf16 blob; with 12-bit slots the compressed blob): the copy engines move the bytes
 *                     and no compute unit takes part, which matters when steps run beside the copies
 *                     (tide_refresh_deferred).
 * Results are identical: the slots end up byte-equal to the host's blobs of the resident form either way. */
#define TIDE_COPY_KERNEL 0
#define TIDE_COPY_DMA    1
int tide_refresh_engine(tide_ctx* ctx, int engine);

/* Policy variant of the counter (the paper clears H at a refresh; Sec. 5 names counters with a longer
 * memory as future work): H[e] <- floor(H[e] * num / den) for every expert of the layer, on hip_stream.
 * Called after tide_refresh(reset_counts = 0) it turns H into an exponentially fading count.
 * 0 <= num <= den, den >= 1 (num == den leaves H as it is: a cumulative counter). */
int tide_scale_counts(tide_ctx* ctx, int layer, int num, int den, void* hip_stream);

/* Snapshot hooks (tests): placement table slot_of[E] (-1 = not resident) to host;
 * raw bytes of a cache slot (slot == capacity: the shared expert) to host. */
int tide_get_table(tide_ctx* ctx, int layer, int32_t* slot_of_host, void* hip_stream);
int tide_read_slot(tide_ctx* ctx, int layer, int slot, void* blob_host);

/* Snapshot hook (tests): how the last tide_moe_step / tide_moe_step_routed on this context cut its hit pairs
 * into grouped-GEMM work items.  Rows are the step's hit pairs (plus one row per token for the shared expert)
 * sorted by cache slot, pairs of one slot in (token, rank) order; row_token_host[r] is the token of row r.  A
 * work item is rows [row0, row0 + nrows) of one slot (slot == capacity: the shared expert); kind 0 = at most 32
 * rows (a slot with more may be cut into several), kind 1 = up to 256 rows of a slot that holds more than 32.
 * At most items_cap / rows_cap entries are written; *n_items_host / *n_rows_host are the full numbers.
 * Synchronises hip_stream.  Not valid after tide_moe_apply_misses (it reuses the lists) or tide_moe_step_noalloc. */
typedef struct { int32_t slot; int32_t row0; int32_t nrows; int32_t kind; } tide_work_item;
int tide_read_work_items(tide_ctx* ctx, tide_work_item* items_host, int items_cap, int* n_items_host,
                         int32_t* row_token_host, int rows_cap, int* n_rows_host, void* hip_stream);

/* Per-call timing of the refresh copies of the LAST tide_refresh on the layer, in
 * milliseconds between the first copy starting and the last one landing; waits for them. */
int tide_refresh_copy_ms(tide_ctx* ctx, int layer, float* ms_out);

/* ---- measurement hooks ---------------------------------------------------------------- */

/* Kernels of one step, in launch order (ids for tide_profile_read). */
#define TIDE_K_ROUTER   0   /* router logits                          */
#define TIDE_K_TOPK     1   /* gate + top-k + hit counts (at <= 32 tokens also the split below, in one workgroup) */
#define TIDE_K_DISPATCH 2   /* hit/miss split, miss list, row lists (own launch above 32 tokens) */
#define TIDE_K_GATE_UP  3   /* grouped gate/up GEMM + SwiGLU          */
#define TIDE_K_DOWN     4   /* grouped down GEMM                      */
#define TIDE_K_COMBINE  5   /* weighted combine                       */
#define TIDE_K_GATE_UP_BIG 6 /* the same two GEMMs over work items of up to 256 rows   */
#define TIDE_K_DOWN_BIG    7 /* (slots with more than 32 rows; not launched at <= 32 tokens) */
#define TIDE_K_COUNT    8

/* enable != 0: from now on every kernel launch of a step carries a start and a stop HIP
 * event that the dispatch itself stamps when it begins and ends on its stream (no extra
 * packets between the kernels).  An event-stamped launch costs the host about 15 us, so a step of
 * five stamped launches can become host-bound; enable == 2 stamps only the expert GEMM launches
 * (TIDE_K_GATE_UP, TIDE_K_DOWN and their _BIG forms), enable == 3 only TIDE_K_GATE_UP(_BIG) and the
 * launch right before it (TIDE_K_TOPK / TIDE_K_DISPATCH).
 * Synchronises the device and drops earlier samples. */
int tide_profile(tide_ctx* ctx, int enable);
/* Waits for the device, then writes per kernel id the summed start-to-stop time in
 * milliseconds (ms_sum_host[TIDE_K_COUNT]) and the number of launches
 * (launches_host[TIDE_K_COUNT]) since the last read, and clears the samples. */
int tide_profile_read(tide_ctx* ctx, double* ms_sum_host, int64_t* launches_host);
/* What this GPU's HBM delivers to a kernel that does nothing but read: the layer's cache slots (capacity +
 * n_shared blobs) are read once per launch, in the access shape of the expert GEMMs' weight stream (whole 1 KiB
 * tiles per wave, non-temporal, eight in flight, two workgroups per compute unit), `repeats` times after one
 * warm-up launch.  *gbytes_per_s_host = bytes per launch / mean launch duration (dispatch-stamped events);
 * *bytes_host (may be NULL) = bytes per launch.  A yardstick for the HBM fractions the step kernels reach:
 * slot sets smaller than the chip's 256 MB memory-side cache read faster than HBM can deliver.
 * Synchronises the device; touches no state. */
int tide_hbm_stream_probe(tide_ctx* ctx, int layer, int repeats, double* gbytes_per_s_host, uint64_t* bytes_host);
/* Running totals kept on the device by the step itself: out4_host = {steps, cache slots
 * (shared expert included) that had at least one token, expert rows evaluated, misses}.
 * Synchronises hip_stream; reset != 0 zeroes them afterwards. */
int tide_counters(tide_ctx* ctx, int64_t* out4_host, int reset, void* hip_stream);

/* ---- refresh-interval analysis (Sec. 3.2; Sec. 3.3 "Interval-based Expert Refresh", Eq. 4-7) ---- */

/* Copies the last step's activation vector -- counts_host[e] = number of tokens that selected
 * expert e in the most recent tide_moe_step / tide_moe_step_routed on this context (Fig. 1a's
 * per-step vectors) -- to host memory.  n_experts must equal the configuration's.  Synchronises
 * hip_stream. */
int tide_step_histogram(tide_ctx* ctx, int32_t* counts_host, int n_experts, void* hip_stream);
/* Routing stability of a run of steps from their activation vectors counts_dev[n_steps][n_experts]
 * (device, int32, row-major).  Any output may be NULL.
 *   sim_dev[n_steps][n_steps] (device, fp64): cosine similarity of steps i and j (Sec. 3.2); a step with
 *     no activations has similarity 0 with every step;
 *   unique_dev[n_steps] (device, int32): distinct experts activated at each step (Fig. 2a);
 *   drift_dev[n_steps] (device, fp64): Eq. 4, d_t = |Delta K_t| / budget, where K_t is the top-`budget`
 *     set of step t's own counts (count descending, lower expert first) and Delta K_t the experts of
 *     K_t that are not in K_{t-1}; d_0 = 0.
 * 1 <= n_experts <= 512, 1 <= budget <= n_experts, n_steps >= 1.  Enqueued on hip_stream, not
 * synchronised.  ctx may be NULL (then errors carry no text). */
int tide_routing_stability(tide_ctx* ctx, const int32_t* counts_dev, int n_steps, int n_experts, int budget,
                           double* sim_dev, int32_t* unique_dev, double* drift_dev, void* hip_stream);
/* The cost model for every candidate interval tau = 1 .. n_steps-1 (host arrays of n_steps-1 doubles):
 *   lat_io_host[tau-1]  = c_io  * (budget * n_steps / tau) * (1 - (1-d)^tau)      (Eq. 5)
 *   lat_cpu_host[tau-1] = c_cpu * n_steps * budget * f_host[tau-1]                (Eq. 6, f_host[tau-1] = f(tau))
 * Pure host arithmetic in fp64; needs no device.  0 <= d <= 1, n_steps >= 2. */
int tide_interval_costs(int budget, int n_steps, double d, double c_io, double c_cpu, const double* f_host,
                        double* lat_io_host, double* lat_cpu_host);
/* Eq. 7 read as min over tau in 1..n_steps-1 of lat_io + lat_cpu, by scanning all candidates (equal totals:
 * the smaller tau): *tau_host = the minimiser, *cost_host = its total.  Host only. */
int tide_optimal_interval(int budget, int n_steps, double d, double c_io, double c_cpu, const double* f_host,
                          int* tau_host, double* cost_host);

/* The constant drift rate for which Eq. 5 reproduces a measured number of migrated experts over n_steps
 * steps at interval tau: *d_host = 1 - (1 - migrations*tau/(budget*n_steps))^(1/tau), the fraction clamped
 * to [0, 1].  Host only. */
int tide_fit_drift(double migrations, int budget, int n_steps, int tau, double* d_host);

#ifdef __cplusplus
}
#endif
#endif /* TIDE_H_ */
