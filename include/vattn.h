/*
 * vattn.h - C ABI of the MI355X (gfx950) contiguous-KV attention library.
 *
 * The library implements the hot path that the vAttention paper (arXiv 2405.04437) speeds up:
 * every request's K and V cache is ONE virtually contiguous tensor; physical memory is mapped under
 * it on demand with the HIP virtual-memory calls, and the attention kernels read K/V with plain
 * pointer arithmetic - there is no block table inside any kernel.
 *
 * Conventions
 *  - All functions are extern "C", take plain pointers and sizes, and return int: >= 0 on success,
 *    -1 on failure (as the paper's step() does).  vattn_last_error() returns a thread-local,
 *    NUL-terminated description of the most recent failure on the calling thread.
 *  - "host" / "device" in a parameter comment says where the pointer must point.
 *  - Index arrays (reqids, cu_q, kv_lens, seq_lens) are HOST pointers; the library validates them
 *    and uploads what the kernels need.  They may be reused as soon as the call returns.
 *  - Q, O, new K/V rows and the decode workspace are DEVICE pointers owned by the caller.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are enqueued,
 *    never synchronised: results are ready when the stream reaches them.
 *  - The library owns all virtual reservations and physical handles from vattn_init() until
 *    vattn_destroy().
 *  - A context is not thread-safe: calls on one context must be serialised by the caller.
 *
 * Notation follows the paper's Table 2: N layers, H KV heads, D head dimension, P bytes per
 * element, B maximum batch size, L maximum context length; Hq query heads (Table 5).
 */
#ifndef VATTN_H
#define VATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vattn_ctx vattn_ctx; /* opaque */

/* Policy for what free_reqid does with a finished request's page-groups: unmap them at once, or keep
 * them mapped for later reuse or reclamation (Sec. 5.3.4; deferred reclamation, Sec. 6.1.2). */
#define VATTN_POLICY_SYNC_UNMAP 0u /* free_reqid unmaps everything at once                      */
#define VATTN_POLICY_DEFERRED 1u   /* pages stay mapped; alloc_reqid prefers the best-backed id;
                                      step() reclaims from inactive ids only when the pool is short */
#define VATTN_POLICY_MASK 0xFu

/* Option bits, or-ed into vattn_config.flags next to the policy. */
#define VATTN_FLAG_BACKGROUND 0x10u     /* Sec. 6.1: after every successful step() a helper thread runs a
                                           background pass while the caller launches the iteration's kernels:
                                           (1) look-ahead - map what lookahead_tokens more tokens per active
                                           request will need (Sec. 6.1.1); under DEFERRED also (2) give pages
                                           of inactive ids back while fewer than reclaim_threshold_page_groups
                                           are free, sparing the id alloc_reqid would return next, and
                                           (3) top that id up to eager_page_groups (Sec. 6.1.2).  The pass is
                                           best effort (what does not fit the free pool is skipped) and is
                                           joined by the next call that reads or changes the bookkeeping, so
                                           the state at every call boundary is deterministic.  With this flag
                                           free_reqid() may only be called once the request's last kernel has
                                           finished: its pages can be unmapped at any time afterwards.      */
#define VATTN_FLAG_STATIC_BACKING 0x20u /* baseline for comparisons: every buffer is fully allocated with
                                           hipMalloc at init (B*S bytes each) and map/unmap only do the
                                           bookkeeping - the static reservation of pre-paging systems       */
#define VATTN_FLAG_TENSOR_SLICING 0x40u /* Discussion section, "tensor slicing": ONE K and ONE V buffer of
                                           shape [B, L, N, H, D]; a page-group holds the tokens of all N
                                           layers, layer n is the slice [:, :, n]; 2 handles per page-group
                                           row instead of 2N, S = L*N*H*D*P                                  */

/* Arguments of init() in Table 4: N, B, L, H, D, P, page-group size (plus what a C library needs). */
typedef struct {
    int32_t num_layers;        /* N                                                               */
    int32_t max_batch;         /* B: reqIds are 0 .. B-1                                          */
    int64_t max_ctx;           /* L: tokens per request the reservation must hold                 */
    int32_t num_q_heads;       /* Hq, a multiple of H                                             */
    int32_t num_kv_heads;      /* H                                                               */
    int32_t head_dim;          /* D: 64 or 128                                                    */
    int32_t elem_bytes;        /* P: 2 (bf16)                                                     */
    int64_t page_group_bytes;  /* 0 = 2 MiB; otherwise a multiple of the granularity reported by
                                  hipMemGetAllocationGranularity                                  */
    int64_t phys_budget_bytes; /* size of the physical page-group pool created at init, summed
                                  over all 2N buffers; rounded down to whole page-groups          */
    int32_t device;            /* HIP device ordinal                                              */
    uint32_t flags;            /* VATTN_POLICY_* | VATTN_FLAG_*                                   */
    int32_t lookahead_tokens;  /* BACKGROUND: tokens of growth mapped ahead of need (1 = next decode
                                  iteration); 0 = none                                            */
    int32_t eager_page_groups; /* BACKGROUND + DEFERRED: page-groups kept mapped under the reqId that
                                  will be handed out next; 0 = none                               */
    int64_t reclaim_threshold_page_groups; /* BACKGROUND + DEFERRED: free-pool level below which
                                  inactive ids give their page-groups back; 0 = never             */
} vattn_config;

/* ---- memory management: Table 4 and Algorithm 1 of the paper -------------------------------- */

/* init (Table 4; Sec. 5.3.1): reserves 2N virtual buffers of B*S bytes each, S = L*H*D*P rounded
 * up to the page-group size (Sec. 5.1.3) - with TENSOR_SLICING, 2 buffers and S = L*N*H*D*P - and
 * creates the physical page-group pool WITHOUT mapping any of it.  *out receives the context.
 * Fails if the device lacks virtual-memory support, the configuration is invalid, the pool cannot
 * be created, or it holds more than 32768 page-groups (larger caches need larger page-groups).
 * Every (buffer, page-group) address that is ever mapped can stay a memory mapping of the process until
 * vattn_destroy(), also after it is unmapped, and Linux caps their number (vm.max_map_count): the
 * library counts them, and step() returns -1 - changing nothing - before that cap would be reached. */
int vattn_init(const vattn_config* cfg /*host*/, vattn_ctx** out /*host*/);

/* Unmaps and releases everything, frees the reservations and the context.  The caller must have
 * synchronised all streams that still use the KV buffers. */
int vattn_destroy(vattn_ctx* ctx);

/* alloc_reqid (Table 4): marks an unused reqId active and returns it, or -1 if all B are in use.
 * SYNC_UNMAP: the lowest unused id.  DEFERRED: the unused id with the most page-groups still
 * mapped (Sec. 6.1.2), ties to the lowest id. */
int vattn_alloc_reqid(vattn_ctx* ctx);

/* free_reqid (Table 4; Sec. 5.3.4): marks reqId inactive.  SYNC_UNMAP: also unmaps all its
 * page-groups in all 2N buffers and returns them to the pool.  DEFERRED: leaves them mapped; a later
 * step() or background pass may take them back.  Under every policy, call it only once the last
 * kernel that reads or writes the request's KV has FINISHED (not merely been enqueued): its pages may
 * be unmapped at any time afterwards.  (step() on the caller's thread additionally waits for the
 * device before it reclaims from inactive ids; SYNC_UNMAP and background passes do not wait.)
 * -1 if reqid is out of range or not active. */
int vattn_free_reqid(vattn_ctx* ctx, int reqid);

/* step (Table 4; Sec. 5.3.3): seq_lens[count], count == B, holds the context length of every
 * reqId (0 for inactive ids).  On return 0, every active request has at least
 * ceil(len*H*D*P / page_group_bytes) page-groups mapped, contiguously from its base, in each of the
 * 2N buffers.  All-or-nothing: if the pool (plus, under DEFERRED, pages held by inactive ids)
 * cannot cover the demand, or an argument is invalid (wrong count, len > L, non-zero length for an
 * inactive id), it returns -1 and changes nothing.  If a driver call fails halfway, everything this
 * call mapped is unmapped again, page-groups it took back from inactive ids are mapped back (they stay
 * in the pool if the driver refuses that as well), and -1 is returned: the mapped counts of the active
 * requests are those at entry.  Lengths that shrink never unmap. */
int vattn_step(vattn_ctx* ctx, const int64_t* seq_lens /*host*/, int count);

/* Request-level indexing (Sec. 5.2.3): device address of reqId's sub-tensor in layer `layer`,
 * which = 0 for K, 1 for V: buffer base + reqId*S.  Layout inside: [L, H, D], token-major; with
 * TENSOR_SLICING [L, N, H, D] and the returned address is that of (token 0, layer), so consecutive
 * tokens of the layer are N*H*D*P bytes apart.  NULL on an invalid argument.  Only the first
 * mapped_page_groups*page_group_bytes bytes of the sub-tensor may be touched. */
void* vattn_kv_ptr(vattn_ctx* ctx, int layer, int which, int reqid);

/* Introspection for tests: active flag, page-groups mapped per sub-tensor (identical in all 2N
 * buffers) and the byte offset reqId*S of the sub-tensor inside each buffer. */
int vattn_query(vattn_ctx* ctx, int reqid, int* active, int64_t* mapped_page_groups, int64_t* va_offset);

/* Page-group size in bytes, S, pool size and free pool count (both in page-groups). */
int vattn_stats(vattn_ctx* ctx, int64_t* page_group_bytes, int64_t* S_bytes, int64_t* pool_total,
                int64_t* pool_free);

/* Cumulative number of (buffer, page-group) map and unmap operations, and the wall time in
 * microseconds the library spent inside hipMemMap+hipMemSetAccess and hipMemUnmap. */
int vattn_counters(vattn_ctx* ctx, int64_t* map_calls, int64_t* unmap_calls, double* map_us, double* unmap_us);

/* Where the mapping work happened (Sec. 6.1, the ablation of Sec. 7.5): map operations done inside
 * step() on the caller's thread vs by background passes, and cumulative microseconds of step()
 * calls, of background passes, and of the caller waiting for a pass to finish.  Any pointer may be
 * NULL. */
int vattn_step_counters(vattn_ctx* ctx, int64_t* sync_map_calls, int64_t* background_map_calls, double* step_us,
                        double* background_us, double* wait_us);

/* Waits for a running background pass (no-op without VATTN_FLAG_BACKGROUND).  Other calls do this by
 * themselves; exposed so that measurements can separate the pass from what follows. */
int vattn_sync(vattn_ctx* ctx);

/* ---- the attention path (Eq. 2 of the paper, evaluated per request) -------------------------- */

/* KV append (Sec. 7.1: with contiguous KV the append is one plain copy): copies the new rows k_new/v_new [sum q_len, H, D]
 * (device, bf16) of n requests to token positions kv_len_before[r] .. kv_len_before[r]+q_len-1 of
 * each request's K and V sub-tensor in `layer`.  cu_q[n+1] are prefix sums of q_len.  The target
 * range must already be mapped by step(). */
int vattn_append_kv(vattn_ctx* ctx, int layer, void* stream, const void* k_new /*device*/,
                    const void* v_new /*device*/, const int32_t* reqids /*host*/,
                    const int32_t* cu_q /*host*/, const int64_t* kv_len_before /*host*/, int n);

/* Causal prefill attention.  q, o: [sum q_len, Hq, D] bf16 (device), packed over the n requests in
 * order; kv_lens[r] is the context length AFTER the q_len newest tokens were appended, so query
 * row i of request r attends to keys 0 .. kv_lens[r]-q_len+i (a chunk appended to an existing
 * context sees all of it).  Query head h reads KV head h/(Hq/H).  scores are multiplied by `scale`
 * (Eq. 2 divides by a constant; pass its reciprocal, 1/sqrt(D) in all workloads here; it must be finite
 * and > 0 in every attention call, else -1).  reqids[r] selects the KV sub-tensor of batch slot r
 * (the batch-index indirection of Sec. 5.3.4).  fp32 accumulation, bf16 output. */
int vattn_attn_prefill(vattn_ctx* ctx, int layer, void* stream, const void* q /*device*/,
                       void* o /*device*/, const int32_t* reqids /*host*/, const int32_t* cu_q /*host*/,
                       const int64_t* kv_lens /*host*/, int n, float scale);

/* Bytes of device workspace vattn_attn_decode needs for these context lengths (split-K partial
 * results).  -1 on an invalid argument. */
int64_t vattn_decode_workspace_bytes(vattn_ctx* ctx, const int64_t* kv_lens /*host*/, int n);

/* Decode attention, one query token per request: q, o [n, Hq, D] bf16 (device).  Runs a split-K
 * kernel over segments of the batch's KV tiles (one per resident workgroup) followed by a reduce kernel that merges the
 * partials of each request (running maximum and sum) and writes bf16.  workspace: device memory
 * of at least vattn_decode_workspace_bytes(), 256-byte aligned, private to this call until the
 * stream has passed it. */
int vattn_attn_decode(vattn_ctx* ctx, int layer, void* stream, const void* q /*device*/,
                      void* o /*device*/, const int32_t* reqids /*host*/, const int64_t* kv_lens /*host*/,
                      int n, float scale, void* workspace /*device*/, size_t workspace_bytes);

/* vattn_attn_decode for callers that cannot allocate device memory or let a library do so: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as
 * vattn_attn_decode without the workspace: the split-K partials live in a device array of 32 MiB that the
 * library owns (one per GPU, held until the process ends), and the call performs no allocation, no copy and
 * no upload - the index arrays travel in the kernel arguments.  Limits, else -1 with a message: n <= 256,
 * and (segments + n) * Hq * (D + 2) * 4 bytes of partials (segments <= CUs + 8) must fit the array - e.g.
 * 256 requests at Hq = 56, D = 128.  Nothing in the array has to start at zero (every slot the reduce
 * kernel reads is written by the split-K kernel of the same call).  All calls on one GPU share the array:
 * calls that may overlap on the device (different streams, or another context on the same GPU) race; keep
 * them on one stream.  Kernel timing (vattn_set_timing) does not cover this entry point. */
int vattn_attn_decode_static(vattn_ctx* ctx, int layer, void* stream, const void* q /*device*/,
                             void* o /*device*/, const int32_t* reqids /*host*/, const int64_t* kv_lens /*host*/,
                             int n, float scale);

/* Decode attention with the KV append fused in (Sec. 7.1 names kernels that write the new K/V rows
 * themselves): k_new, v_new [n, H, D] bf16 (device) are the K/V rows of each request's NEWEST token;
 * kv_lens[r] counts that token (it is position kv_lens[r]-1, which step() must already have mapped).
 * The kernel stores the rows into the cache of `layer` and attends over all kv_lens[r] tokens; the
 * result equals vattn_append_kv followed by vattn_attn_decode.  A reqId may appear only once. */
int vattn_attn_decode_append(vattn_ctx* ctx, int layer, void* stream, const void* q /*device*/,
                             const void* k_new /*device*/, const void* v_new /*device*/, void* o /*device*/,
                             const int32_t* reqids /*host*/, const int64_t* kv_lens /*host*/, int n, float scale,
                             void* workspace /*device*/, size_t workspace_bytes);

/* Prefill with the KV append fused in (which the paper's Sec. 7.1 leaves as a separate copy).  k_new, v_new: [sum q_len, H, D] bf16 (device), the K/V rows of the query tokens, packed
 * like q; they are NOT in the cache yet.  kv_lens[r] counts them (positions kv_lens[r]-q_len .. kv_lens[r]-1,
 * which step() must already have mapped).  One launch stores the rows into the cache of `layer` and attends;
 * the result equals vattn_append_kv (kv_len_before = kv_lens - q_len) followed by vattn_attn_prefill.  A reqId
 * with a non-empty chunk may appear only once. */
int vattn_attn_prefill_append(vattn_ctx* ctx, int layer, void* stream, const void* q /*device*/,
                              const void* k_new /*device*/, const void* v_new /*device*/, void* o /*device*/,
                              const int32_t* reqids /*host*/, const int32_t* cu_q /*host*/,
                              const int64_t* kv_lens /*host*/, int n, float scale);

/* Comparison kernel, not part of the method: the SAME split-K decode over a PAGED KV cache, the design
 * the paper argues against (Sec. 3: block table inside the kernel), to re-measure on this GPU what the
 * indirection costs.  k_pool, v_pool: caller-owned device pools [num_blocks, block_tokens, H, D] bf16;
 * block_table [n, max_blocks_per_req] (HOST; validated and uploaded): entry j of row r names the block
 * that holds tokens j*block_tokens .. of batch slot r.  block_tokens: a multiple of 32.  The context
 * only supplies the head geometry; its own KV buffers are not touched.  Same workspace rule as
 * vattn_attn_decode (vattn_decode_workspace_bytes with the same kv_lens). */
int vattn_attn_decode_paged(vattn_ctx* ctx, void* stream, const void* q /*device*/, void* o /*device*/,
                            const void* k_pool /*device*/, const void* v_pool /*device*/, int64_t num_blocks,
                            int block_tokens, const int32_t* block_table /*host*/, int max_blocks_per_req,
                            const int64_t* kv_lens /*host*/, int n, float scale, void* workspace /*device*/,
                            size_t workspace_bytes);

/* The same comparison for prefill: the default prefill kernel with a block-table lookup per 64-token
 * tile.  Arguments as for vattn_attn_decode_paged and vattn_attn_prefill; block_tokens: a multiple of 64;
 * kv_lens[r] counts the query tokens, which must already be in the pools. */
int vattn_attn_prefill_paged(vattn_ctx* ctx, void* stream, const void* q /*device*/, void* o /*device*/,
                             const void* k_pool /*device*/, const void* v_pool /*device*/, int64_t num_blocks,
                             int block_tokens, const int32_t* block_table /*host*/, int max_blocks_per_req,
                             const int32_t* cu_q /*host*/, const int64_t* kv_lens /*host*/, int n, float scale);

/* ---- measurement helpers --------------------------------------------------------------------- */

/* When enabled, every launch of the split-K decode kernel, the reduce kernel, the prefill kernel and the
 * KV-append kernel carries a pair of HIP events that the launch stream records when the kernel starts and when it
 * ends (hipExtLaunchKernelGGL), so their distance is the kernel's execution time without launch
 * gaps; vattn_kernel_time() then synchronises those events and returns the accumulated kernel time
 * in milliseconds and the number of launches since the last call, per kernel (which: 0 = decode
 * split-K, 1 = prefill, 2 = decode reduce, 3 = KV append), and resets them. */
int vattn_set_timing(vattn_ctx* ctx, int enabled);
int vattn_kernel_time(vattn_ctx* ctx, int which, double* total_ms, int64_t* launches);

/* Tuning knobs of the split-K decode.  By default the library cuts the batch's 32-token tiles into as
 * many segments as one launch keeps resident on the chip (one workgroup of four waves per CU), with
 * lengths proportional to a weight per XCD (segment s runs on XCD s % 8).  set_decode_chunk fixes one
 * segment length instead (tokens, a multiple of 32; 0 = default).  set_decode_tuning chooses how many
 * segments are cut per resident workgroup slot (>= 1; 1 measured best).  set_decode_xcd_weights replaces
 * the eight weights (host array, each in [0.25, 4]; NULL restores the default 1, 0.9, 1, 0.9, ... -
 * measured on MI355X: the odd XCDs draw about 10 % less bandwidth).  Results are identical up to
 * floating-point summation order. */
int vattn_set_decode_chunk(vattn_ctx* ctx, int tokens);
int vattn_set_decode_tuning(vattn_ctx* ctx, int segments_per_slot);
int vattn_set_decode_xcd_weights(vattn_ctx* ctx, const float* weights /*host, 8 values, or NULL*/);

const char* vattn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* VATTN_H */
