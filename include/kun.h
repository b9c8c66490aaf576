/*
 * kun.h -- C ABI of the MI355X (gfx950) paged-attention library.
 *
 * The library implements the attention step of one transformer layer over a block-table KVCache
 * whose block pool can grow at run time: batched decode and chunked prefill.  It is the kernel a
 * serving instance runs after a parameter drop has handed freed parameter memory to the KVCache
 * (KunServe, Section 3 and Section 4.1 "Local instance memory management"): requests, fixed-size
 * KV blocks and per-request block tables, with the pool described as a list of byte ranges -- the
 * first pool plus one range per extension -- instead of the single static
 * [base, base + num_blocks * block_size] layout that Section 4.1 says existing kernels assume.
 *
 * Conventions for every call
 *   - Return value: a kun_status (0 = KUN_OK, negative = error).  Argument errors are found on
 *     the host before anything is launched; no call leaves a partial launch behind.
 *   - "device" pointers are HIP device addresses; "host" pointers are ordinary process memory.
 *   - The caller owns every buffer it passes (pool ranges, q, out, tables, workspace) and keeps
 *     it alive until the work enqueued on `stream` has finished; the library owns only the small
 *     host object behind kun_kv_pool.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  kun_kv_append,
 *     kun_paged_decode and kun_paged_prefill_chunk only enqueue kernels: they do not synchronise,
 *     allocate or free.
 *   - Physical block ids are int32, cumulative over the ranges in the order the ranges were
 *     added, and never renumbered.  Block-table entries at or beyond ceil(L / block_size) of a
 *     request are ignored and may hold anything (e.g. -1).  Ids the kernels do read must be
 *     valid: check tables with kun_validate_block_table when in doubt.  (An id outside the pool is
 *     not followed: the attention kernels clamp it into [0, num_blocks), so the request it belongs
 *     to reads some other block of the pool and its output means nothing, but no address outside
 *     the pool's ranges is touched; kun_kv_append leaves such a token out.)
 *
 * Page layout (part of the ABI).  One block is num_kv_heads pages; page (block, kv head) is
 *   block_size / 16 tiles in token order, and the tile of tokens 16 i .. 16 i + 15 is
 *     K  [16 tokens][head_dim]      then
 *     V  [head_dim][16 tokens]      (V is stored transposed inside a tile)
 *   (a page of 64 tokens is laid out as four pages of 16 tokens in a row: every kernel reads whole,
 *   contiguous tiles whatever the block size), so
 *   block_bytes = 2 * num_kv_heads * block_size * head_dim * sizeof(element); with 8 KV heads of
 *   128 dims in bf16 that is 4096 bytes per token per layer, the figure behind the 192 KB per
 *   token of a 48-layer model quoted in Section 2.2.
 *   Query heads h with the same h / (num_q_heads / num_kv_heads) share a KV head (GQA).
 *
 * Supported shapes: block_size 16, 32, 64 or 128 (Section 5.1 tunes it to 64); head_dim 64 or 128;
 *   num_q_heads / num_kv_heads = 1 .. 8 (e.g. 40 query heads over 8 KV heads), or 16 with bf16 and
 *   head_dim 128 (e.g. 64 over 4); dtype f32, bf16 or FP8 E4M3 pages with bf16 queries
 *   (accumulation is always fp32).  Anything else is KUN_ERR_UNSUPPORTED.  bf16 with head_dim 128
 *   runs on the matrix cores (decode and prefill), and so do FP8 pages with head_dim 128 (16 query
 *   heads per KV head included); the other combinations run on vector-ALU kernels that are correct
 *   to the same bar but not tuned.
 */
#ifndef KUN_H
#define KUN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KUN_API __attribute__((visibility("default")))

typedef struct kun_kv_pool kun_kv_pool; /* opaque host object */

/* Element type of the K/V pages.  KUN_FP8_E4M3: pages hold OCP FP8 E4M3 codes (1 sign, 4 exponent bits
 * with bias 7, 3 mantissa bits, no infinities, NaN = S.1111.111), one byte per element -- the lossy KV
 * representation Section 7 names as the alternative under memory pressure; queries, outputs and the
 * softmax weights fed to the matrix cores stay bf16, accumulation fp32, and the K/V rows handed to
 * kun_kv_append are FP8 bytes already (the caller quantises). */
typedef enum { KUN_F32 = 0, KUN_BF16 = 1, KUN_FP8_E4M3 = 2 } kun_dtype;

typedef enum {
    KUN_OK = 0,
    KUN_ERR_INVALID_ARG = -1,     /* null pointer, non-positive size, heads not divisible, ...  */
    KUN_ERR_MISALIGNED = -2,      /* a range base that is not 256-byte aligned                  */
    KUN_ERR_TOO_SMALL = -3,       /* a range smaller than one block                             */
    KUN_ERR_TOO_MANY_RANGES = -4, /* more than KUN_MAX_RANGES ranges                            */
    KUN_ERR_BLOCK_OOB = -5,       /* a block id outside [0, num_blocks)                         */
    KUN_ERR_WORKSPACE = -6,       /* workspace missing, misaligned or smaller than required     */
    KUN_ERR_HIP = -7,             /* a HIP launch failed                                        */
    KUN_ERR_UNSUPPORTED = -8,     /* shape or dtype outside the supported set                   */
    KUN_ERR_OVERLAP = -9,         /* a new range overlaps one already in the pool               */
    KUN_ERR_SCRATCH_LIMIT = -10   /* the call needs more than the library's fixed scratch array */
} kun_status;

#define KUN_MAX_RANGES 16

/* Human-readable name of a status code (static storage). */
KUN_API const char* kun_status_string(int status);

/* After a call on this host thread returned KUN_ERR_HIP: which HIP call failed and the driver's
 * message for it ("" if none has failed yet).  The string is owned by the library and overwritten
 * by the next failure on the same thread. */
KUN_API const char* kun_last_hip_error(void);

/* Tuning options for tests and sweeps, process-wide.  The library reads the environment variables of
 * the same names ONCE, when it is loaded; afterwards only this call changes an option (value NULL or
 * "" = back to the default), and no launch reads the environment.  Not synchronised with launches
 * made from other host threads.  KUN_ERR_INVALID_ARG for an unknown name or a value outside the set:
 *   KUN_DECODE_PART    tokens per split-K partition, a multiple of 32 (default: chosen from the bound)
 *   KUN_DECODE_WAVES   1, 2 or 4 waves per workgroup of the matrix-core decode kernel (default 4)
 *   KUN_DECODE_KERNEL  "generic": the vector-ALU decode kernel for every shape; "mfma": the default
 *   KUN_DECODE_MAP     "flat": item-major workgroup order; "xcd": the default XCD-aware order
 *   KUN_DECODE_MERGE   "fold": partial results are merged inside the partial kernel; "kernel": by a launch
 *                      of its own; "auto": by batch size (the default)
 *   KUN_PREFILL_SHAPE  "persistent": workgroups that fetch their work items, one per compute unit;
 *                      "ring": the one-barrier-per-tile kernel (cross-check), "ring-persistent"; "default" */
KUN_API int kun_set_option(const char* name, const char* value);

/* ---- pool growth (Section 4.1: the KVCache region is extended at its tail with the memory of
 *      dropped parameters; Section 5.6: two consecutive drops enlarge it twice) ---------------- */

/* Create a pool whose first range is the device byte range [base, base + bytes).
 * Usable blocks = floor(bytes / block_bytes); the remainder is unused.  Host-only. */
KUN_API int kun_kv_pool_create(kun_kv_pool** out, void* base, size_t bytes, int dtype, int num_kv_heads,
                       int head_dim, int block_size);

/* Append the device byte range [base, base + bytes) -- e.g. the buffer of a dropped parameter --
 * as a new range.  Existing block ids, addresses and contents are untouched; the new blocks get
 * ids first_new_block .. first_new_block + num_new_blocks - 1 (both optional outputs, host).
 * Takes effect for calls issued after it returns; kernels already enqueued keep the table they
 * were launched with.  Host-only, no device work. */
KUN_API int kun_kv_pool_extend(kun_kv_pool* pool, void* base, size_t bytes, int64_t* first_new_block,
                       int64_t* num_new_blocks);

/* The LAST range of the pool now spans new_bytes from its unchanged base: it grew in place (memory
 * was mapped behind it, see kun_vmm_region below) or lost its tail (restoration).  Blocks that stay
 * keep their ids and addresses; new blocks continue the numbering; after a shrink the ids from
 * *first_changed_block on no longer exist, and it is the caller's job that no table still names
 * them and no enqueued work still reads them.  *first_changed_block: first id added or removed;
 * *num_blocks_delta: blocks added (> 0) or removed (< 0).  Outputs optional. */
KUN_API int kun_kv_pool_resize_tail(kun_kv_pool* pool, size_t new_bytes, int64_t* first_changed_block,
                            int64_t* num_blocks_delta);

KUN_API int kun_kv_pool_num_blocks(const kun_kv_pool* pool, int64_t* n);
KUN_API int kun_kv_pool_num_ranges(const kun_kv_pool* pool, int* n);
KUN_API int kun_kv_pool_block_bytes(const kun_kv_pool* pool, size_t* bytes);

/* Block id -> range index, byte offset inside that range, device address (outputs optional).
 * This is the address arithmetic the kernels apply to every table entry. */
KUN_API int kun_kv_pool_resolve(const kun_kv_pool* pool, int64_t block, int* range, size_t* byte_off,
                        void** addr);

/* Frees the host object only; never touches the ranges. */
KUN_API int kun_kv_pool_destroy(kun_kv_pool* pool);

/* Host-side check of a HOST copy of a block table [rows, max_blocks] against HOST context lengths
 * [rows]: every entry below ceil(len / block_size) must be in [0, num_blocks) and len must fit
 * max_blocks.  Returns KUN_ERR_BLOCK_OOB / KUN_ERR_INVALID_ARG on the first violation. */
KUN_API int kun_validate_block_table(const kun_kv_pool* pool, const int32_t* host_table, int rows,
                             int max_blocks, const int32_t* host_ctx_len);

/* Device-side view of block resolution (section 4.1: blocks that live in the remapped tail of the
 * KV region are addressed like any other).  For each of T (row, position) pairs -- device int32
 * arrays as in kun_kv_append -- a kernel walks block_table (device int32 [rows, max_blocks]) and
 * the range table exactly as the attention kernels do and writes, for KV head kv_head:
 *   range_out[i]  index of the range that holds the token's block          (device int32 [T])
 *   k_off_out[i]  byte offset inside that range of K[position][0]          (device int64 [T])
 *   v_off_out[i]  byte offset inside that range of V[position][0]; element j of the V row sits
 *                 j * 16 elements further on (the tile's row stride)       (device int64 [T])
 * Integer outputs, exact; all three are -1 for a pair the table cannot place (see kun_kv_append).
 * T == 0 is a no-op. */
KUN_API int kun_slot_map(const kun_kv_pool* pool, const int32_t* seq_of_tok, const int32_t* pos_of_tok,
                 int T, const int32_t* block_table, int max_blocks, int kv_head,
                 int32_t* range_out, int64_t* k_off_out, int64_t* v_off_out, void* stream);

/* ---- KV append: write the K/V rows of new tokens into their slots -------------------------- */

/* k_new, v_new: device [T, num_kv_heads, head_dim] in the pool's dtype (FP8 pools: one byte per element).  Token i belongs to row
 * seq_of_tok[i] of block_table (device int32 [rows, max_blocks]) at logical position
 * pos_of_tok[i] (device int32 [T]); it lands in block block_table[seq][pos / block_size], slot
 * pos % block_size.  T == 0 is a no-op.  Checked on the device, without an error code: a token whose
 * row or position is below zero, whose position is beyond the max_blocks * block_size tokens of a table
 * row, or whose table entry is not a block of the pool (e.g. -1) is left out -- nothing is written for
 * it.  (The number of table rows is not known to the call: a row index beyond the table is the
 * caller's to avoid.) */
KUN_API int kun_kv_append(kun_kv_pool* pool, const void* k_new, const void* v_new,
                  const int32_t* seq_of_tok, const int32_t* pos_of_tok, int T,
                  const int32_t* block_table, int max_blocks, void* stream);

/* ---- batched decode ------------------------------------------------------------------------ */

/* Bytes of device workspace kun_paged_decode needs for S requests whose context lengths sum to at
 * most total_ctx_upper_bound tokens (pass 0 to assume a full pool).  0 on bad arguments. */
KUN_API size_t kun_decode_workspace_bytes(const kun_kv_pool* pool, int S, int num_q_heads,
                                  int64_t total_ctx_upper_bound);

/* One decode step for S requests (Section 2.1: decode reads the whole KVCache of each request
 * and is memory-bound).  q, out: device [S, num_q_heads, head_dim] in the pool's dtype (bf16 for FP8 pools); request s
 * has ctx_len[s] tokens in its pages INCLUDING the token being decoded, whose query is row s of q;
 * out[s] = softmax(scale * q K^T) V over those tokens.  ctx_len: device int32 [S]; a request with
 * ctx_len 0 (or below, or above the max_blocks * block_size tokens its table row can hold) is
 * skipped and its output row left untouched.  block_table: device int32
 * [S, max_blocks].  total_ctx_upper_bound: host-known bound on sum(ctx_len) (0 = full pool); it
 * sizes the launch and must be the value used for kun_decode_workspace_bytes or smaller; the
 * split-K partition size is chosen from it, so a bound close to the real sum is faster than 0.  If
 * sum(ctx_len) is above it, the requests whose partial results no longer fit the workspace are
 * left out as a whole (their rows of out stay untouched); nothing is read or written out of bounds.
 * workspace: device, 256-byte aligned, holds the split-K partial results; contents are scratch. */
KUN_API int kun_paged_decode(kun_kv_pool* pool, const void* q, void* out, const int32_t* block_table,
                     int max_blocks, const int32_t* ctx_len, int S, int num_q_heads, float scale,
                     int64_t total_ctx_upper_bound, void* workspace, size_t workspace_bytes,
                     void* stream);

/* kun_paged_decode in two steps, for callers that decode the same batch more than once: the work list
 * of a decode step (which partitions of which request's context a workgroup reads, and where its
 * partial result goes) depends on the context lengths only, not on q, the pages or the block ids, so
 * a serving step makes it once and every layer of the model runs against it (Section 2.1: one
 * batch passes through all layers).  kun_decode_plan writes the list into the workspace (one small
 * launch); kun_paged_decode_planned is kun_paged_decode without that launch.  Between the two, and
 * between one planned call and the next, the first kun_decode_workspace_bytes-sized part of the
 * workspace must be left alone; a planned call must be given the ctx_len contents, S, num_q_heads and
 * total_ctx_upper_bound of the plan and a pool with the plan's pool's num_kv_heads, head_dim and
 * dtype (the pool itself, its blocks and the block table may differ: another layer's cache).
 * Planned calls on one workspace must not overlap in time.  Results are those of kun_paged_decode
 * bit for bit.  The plan leaves a tag of its batch shape in the workspace; a planned call that does not
 * find the tag it expects (no plan, the plan of another S / bound / head count) launches kernels that
 * compute nothing, and out is left as it was -- no error is returned, the check is on the device.  A
 * plan of the same shape made for other lengths cannot be told apart: the call then computes the
 * attention of the plan's lengths (list entries longer than the block table covers are skipped). */
KUN_API int kun_decode_plan(kun_kv_pool* pool, const int32_t* ctx_len, int S, int num_q_heads,
                    int64_t total_ctx_upper_bound, void* workspace, size_t workspace_bytes, void* stream);
KUN_API int kun_paged_decode_planned(kun_kv_pool* pool, const void* q, void* out, const int32_t* block_table,
                             int max_blocks, const int32_t* ctx_len, int S, int num_q_heads, float scale,
                             int64_t total_ctx_upper_bound, void* workspace, size_t workspace_bytes,
                             void* stream);

/* kun_paged_decode for callers that cannot allocate a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same operation, arguments, kernels and results,
 * but the split-K records go to a fixed array of KUN_STATIC_SCRATCH_BYTES inside the library's device
 * image -- every GPU the library is used on holds its own copy until the process ends -- and the call
 * allocates and frees nothing.  KUN_ERR_SCRATCH_LIMIT if
 * kun_decode_workspace_bytes(pool, S, num_q_heads, total_ctx_upper_bound) exceeds that size (nothing
 * is launched then); pass a tight bound, since 0 sizes for a full pool.  All calls on one GPU share
 * the one array: calls that overlap in time on the same GPU (two streams, two host threads) race;
 * calls in sequence on one stream are safe, nothing is carried over from one call to the next.  The
 * first call on a device looks the array's address up (hipGetSymbolAddress); make it outside any
 * stream capture. */
#define KUN_STATIC_SCRATCH_BYTES (32u << 20)
KUN_API int kun_paged_decode_static(kun_kv_pool* pool, const void* q, void* out, const int32_t* block_table,
                            int max_blocks, const int32_t* ctx_len, int S, int num_q_heads, float scale,
                            int64_t total_ctx_upper_bound, void* stream);

/* ---- chunked prefill ----------------------------------------------------------------------- */

/* Bytes of device workspace kun_paged_prefill_chunk needs for n_chunks chunks holding
 * total_new_tokens query rows in total, with a block table of max_blocks entries per chunk (the
 * workspace holds, among other things, the resolved address of every block a chunk can name). */
KUN_API size_t kun_prefill_workspace_bytes(const kun_kv_pool* pool, int n_chunks, int num_q_heads,
                                   int total_new_tokens, int max_blocks);

/* Attention for n_chunks prefill chunks (Section 4.3, Eq. 1: chunk j of a request has c new tokens
 * after p prior tokens; it attends to the p prior tokens and causally to itself, diagonal
 * included, p*c + (c*c + c)/2 pairs).  The K/V of the chunk's own tokens must already be in the
 * pages (kun_kv_append).  q, out: device [total_new_tokens, num_q_heads, head_dim], chunks packed
 * back to back; q_start: device int32 [n_chunks + 1], row offsets with q_start[n_chunks] ==
 * total_new_tokens; prior_len: device int32 [n_chunks]; block_table: device int32
 * [n_chunks, max_blocks], row i covering the p_i + c_i tokens of chunk i's request.  Row r of
 * chunk i sees logical keys 0 .. p_i + r.  A chunk with c == 0 is skipped, and so is -- checked on the
 * device, no error is returned -- a chunk whose lengths do not fit together: rows outside
 * [0, total_new_tokens), c_i < 0, p_i < 0, or p_i + c_i beyond the max_blocks * block_size tokens its
 * table row can hold; its rows of out stay untouched and nothing is read on its behalf.
 * bf16 and FP8 pools with
 * head_dim 128 run on the matrix cores (q, out of FP8 pools: bf16); fp32 and head_dim 64 pools are
 * served row by row by the vector-ALU decode kernel (correct to the same bar, not tuned). */
KUN_API int kun_paged_prefill_chunk(kun_kv_pool* pool, const void* q, void* out, const int32_t* q_start,
                            const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                            int n_chunks, int num_q_heads, int total_new_tokens, float scale,
                            void* workspace, size_t workspace_bytes, void* stream);

/* kun_paged_prefill_chunk in two steps.  kun_prefill_plan makes the call's work list and resolves the
 * block table into page addresses (one small launch; it reads q_start, prior_len, block_table and the
 * pool's ranges, not q or the pages, so it can be enqueued before the kun_kv_append of the same step,
 * or on another stream while the layer before runs); kun_paged_prefill_chunk_planned is the rest of
 * the call and finds that plan in the workspace.  Unlike a decode plan it holds addresses: it serves
 * this pool as it is (extending the pool afterwards is fine, moving its tail is not) and this block
 * table; the planned call takes the same q_start, prior_len, block_table, max_blocks, n_chunks,
 * num_q_heads and total_new_tokens, and the workspace must be left alone in between.  Results are
 * those of kun_paged_prefill_chunk bit for bit; a planned call that does not find the tag of a plan of
 * its batch shape computes nothing and leaves out as it was.  Pools served row by row (fp32,
 * head_dim 64) plan inside the planned call; kun_prefill_plan is a no-op for them. */
KUN_API int kun_prefill_plan(kun_kv_pool* pool, const int32_t* q_start, const int32_t* prior_len,
                     const int32_t* block_table, int max_blocks, int n_chunks, int num_q_heads,
                     int total_new_tokens, void* workspace, size_t workspace_bytes, void* stream);
KUN_API int kun_paged_prefill_chunk_planned(kun_kv_pool* pool, const void* q, void* out, const int32_t* q_start,
                                    const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                                    int n_chunks, int num_q_heads, int total_new_tokens, float scale,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* Mixed batches (Section 2.1: prefill is compute-bound, decode memory-bound, and serving systems
 * batch the two): the same operation, results and workspace as kun_paged_prefill_chunk, but run by
 * at most max_workgroups workgroups (> 0; rounded down to a multiple of 8, at least 8) that fetch
 * the work items themselves.  One such workgroup fills a compute unit, so enqueuing this call on
 * one stream and kun_paged_decode on another leaves the other compute units to the decode kernel
 * and the two overlap instead of running back to back.  The two calls need separate workspaces. */
KUN_API int kun_paged_prefill_chunk_on(kun_kv_pool* pool, const void* q, void* out, const int32_t* q_start,
                               const int32_t* prior_len, const int32_t* block_table, int max_blocks,
                               int n_chunks, int num_q_heads, int total_new_tokens, float scale,
                               int max_workgroups, void* workspace, size_t workspace_bytes, void* stream);

/* ---- the KVCache region as ONE growing virtual range (Section 4.1) -------------------------- */

/* Section 4.1 keeps attention kernels unchanged by reserving one virtual address range for the
 * largest KVCache, mapping physical memory at its tail as the pool grows and remapping the
 * physical memory of dropped parameters there without a copy; Section 4.4 moves it back when the
 * parameters are restored.  A kun_vmm_region is such a range on the current device.  All calls are
 * host calls that change address mappings: the caller synchronises first with any enqueued work
 * that touches the bytes being unmapped.  Sizes passed to grow are multiples of the region's
 * granularity; sizes passed to move_tail / shrink must add up to whole chunks at the tail (a chunk
 * = the bytes of one grow call): KUN_ERR_MISALIGNED otherwise.  KUN_ERR_TOO_SMALL: reservation
 * exhausted.  KUN_ERR_HIP: the driver refused (e.g. out of memory). */
typedef struct kun_vmm_region kun_vmm_region;

/* Reserve reserve_bytes (rounded up to the granularity) of virtual addresses; nothing is mapped. */
KUN_API int kun_vmm_region_create(kun_vmm_region** out, size_t reserve_bytes);
/* base: device address of the range; mapped_bytes: [base, base + mapped_bytes) is usable memory. */
KUN_API int kun_vmm_region_info(const kun_vmm_region* region, void** base, size_t* mapped_bytes,
                        size_t* reserved_bytes, size_t* granularity);
/* Allocate `bytes` of device memory as one chunk and map it at the tail. */
KUN_API int kun_vmm_region_grow(kun_vmm_region* region, size_t bytes);
/* Unmap the last `bytes` of src (whole chunks) and map the same physical chunks, in the same order,
 * at the tail of dst: the contents move with them, no copy is made.  All or nothing: when a driver
 * call fails (KUN_ERR_HIP) the steps already made are undone and both regions are what they were.
 * Should the driver refuse the undoing as well, both regions still list exactly what is mapped -- src
 * ends below the first chunk that could not be put back, dst keeps the chunks that arrived, a chunk
 * mapped nowhere is released -- and kun_vmm_region_info shows it (mapped_bytes changed). */
KUN_API int kun_vmm_region_move_tail(kun_vmm_region* src, kun_vmm_region* dst, size_t bytes);
/* Unmap the last `bytes` and give the physical memory back to the driver. */
KUN_API int kun_vmm_region_shrink(kun_vmm_region* region, size_t bytes);
/* Unmaps and releases whatever is still mapped, then frees the reservation and the object. */
KUN_API int kun_vmm_region_destroy(kun_vmm_region* region);

/* ---- host-side planning around the attention path ------------------------------------------ */

/* Cost model of Section 4.3.  Eq. 1: a chunk of `tokens` new tokens after `prior` tokens of the same
 * request costs alpha * (prior * tokens + (tokens^2 + tokens) / 2) + beta * tokens + gamma (prefix
 * attention, causal self attention, per-token work, per-launch rest).  Eq. 2-3: a microbatch costs
 * the sum over its chunks with tokens > 0 minus (n - 1) * gamma, the parameters being loaded once. */
typedef struct kun_cost_model { double alpha, beta, gamma; } kun_cost_model;
typedef struct kun_chunk { int32_t request, prior, tokens; } kun_chunk;

/* NaN on bad arguments. */
KUN_API double kun_cost_chunk(const kun_cost_model* model, int64_t prior, int64_t tokens);
KUN_API double kun_cost_microbatch(const kun_cost_model* model, const kun_chunk* chunks, int n);

/* Least-squares fit of the three constants to measured times (offline profiling, Section 4.3):
 * microbatch k consists of host chunks[mb_start[k] .. mb_start[k + 1]) and took seconds[k].
 * KUN_ERR_INVALID_ARG if fewer than 3 microbatches are given or they do not determine the model. */
KUN_API int kun_cost_fit(const kun_chunk* chunks, const int32_t* mb_start, int n_microbatches,
                 const double* seconds, kun_cost_model* out);

/* Lookahead batch formulation (Section 4.3): the queued chunks (host array, queue order, one entry
 * per request with its tokens still to run after `prior`) start as ONE microbatch, which is split
 * recursively into two microbatches of as equal cost as a cut at a token boundary allows -- a cut
 * request continues in the right half with a larger `prior` -- level by level, until a split would
 * leave a side with fewer than min_tokens tokens or the next level would exceed max_microbatches
 * (0 = no limit).  Writes the microbatches back to back into out_chunks (capacity
 * chunk_capacity) with out_mb_start[k] .. out_mb_start[k + 1] delimiting microbatch k (capacity
 * mb_capacity microbatches, mb_capacity + 1 entries).  KUN_ERR_TOO_SMALL if a capacity does not
 * suffice; the constants of the model must be >= 0. */
KUN_API int kun_lookahead(const kun_cost_model* model, const kun_chunk* queue, int n, int min_tokens,
                  int max_microbatches, kun_chunk* out_chunks, int chunk_capacity,
                  int32_t* out_mb_start, int mb_capacity, int* n_microbatches, int* n_chunks);

/* Drop-plan generation (Section 4.1, "Parameter drop during memory overloading", Algorithm 1): instance groups, each holding one copy of the num_layers
 * layers, wait in a priority queue by size (equal sizes: the group formed first); while
 * demand_bytes is not met and two groups remain, the two smallest merge and one redundant copy
 * (num_layers * layer_bytes) is dropped.  initial_group: host [n_instances], group number of each
 * instance before the plan (NULL = every instance alone).  Outputs, host arrays [n_instances]:
 * group_of_instance (final groups numbered by their smallest instance), kept_first / kept_end (the
 * contiguous layers [first, end) the instance keeps: the j-th smallest instance of a group of g is
 * pipeline stage j and keeps layers floor(j L / g) .. floor((j + 1) L / g) - 1), dropped_bytes
 * (what it can hand to its KVCache: kun_kv_pool_extend or kun_vmm_region_move_tail).  Optional
 * [2 * (n_instances - 1)]: merge_members (one instance of each of the two groups of every merge,
 * in order) and merge_sizes.  *demand_met == 0 means no plan frees enough: fall back. */
KUN_API int kun_drop_plan(int n_instances, const int32_t* initial_group, int num_layers, int64_t layer_bytes,
                  int64_t demand_bytes, int32_t* group_of_instance, int32_t* kept_first,
                  int32_t* kept_end, int64_t* dropped_bytes, int32_t* merge_members,
                  int32_t* merge_sizes, int* n_merges, int64_t* freed_bytes, int* demand_met);

#ifdef __cplusplus
}
#endif
#endif /* KUN_H */
