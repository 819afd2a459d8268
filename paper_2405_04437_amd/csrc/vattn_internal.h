// Internal declarations shared by the translation units of libvattn (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/vattn.h"
#include "../../include/vattn_bench.h"
#include "decode_plan.h"
#include "prefill_plan.h"
#include "kv_memory.h"

namespace vattn {

bool hip_ok(hipError_t e, const char* what);  // records the error text and returns false on failure

// Driver-operation tables for the memory manager: HIP virtual-memory calls, and the statically backed
// baseline (whole buffers from hipMalloc, mapping reduced to bookkeeping).
const VmmOps& hip_vmm_ops();
const VmmOps& hip_static_ops();
bool vmm_microbench(int device, int64_t bytes, int count, double* out_us);
bool mfma_microbench(int device, int mode, int rounds, double* tflops, double* shader_mhz);
bool stream_microbench(int device, int64_t bytes, double* gbs);

// ---------------------------------------------------------------------------------------------
// Pinned staging ring for the small index arrays every attention call uploads.
// ---------------------------------------------------------------------------------------------
class MetaRing {
public:
    ~MetaRing();
    // Returns a host pointer (pinned) of at least `bytes` bytes and its device mirror.
    bool acquire(size_t bytes, char** host, char** dev);
    // Enqueues the upload of the first `bytes` bytes of the acquired slot on `stream`.
    bool commit(size_t bytes, hipStream_t stream);
    // Call after the last kernel that reads the slot's device mirror has been enqueued on `stream`: moves the
    // slot's event behind those kernels, so that the slot is only handed out again (eight acquisitions later,
    // possibly for a call on another stream) once they have finished - not merely once the upload has.
    bool release(hipStream_t stream);

private:
    static constexpr int kSlots = 8;
    bool grow(size_t bytes);
    char* host_ = nullptr;
    char* dev_ = nullptr;
    size_t slot_bytes_ = 0;
    int cur_ = -1;
    hipEvent_t ev_[kSlots] = {};
    bool pending_[kSlots] = {};
};

struct KernelTimer {
    struct Pair { hipEvent_t a, b; };
    std::vector<Pair> open;    // recorded, not yet read
    std::vector<Pair> spare;   // reusable events
    // Hands out the event pair of the next launch; the launcher attaches both to the kernel's dispatch,
    // so their distance is the kernel's own execution time (no launch gaps, no neighbouring commands).
    bool next(hipEvent_t* start, hipEvent_t* stop);
    bool collect(double* total_ms, int64_t* launches);
    void destroy();
};

// ---------------------------------------------------------------------------------------------
// Kernel launchers (one per .hip file).  All pointers are device pointers.
// ---------------------------------------------------------------------------------------------
// Optional events recorded at the start and at the end of the kernel itself (both null: not timed).
struct LaunchEvents { hipEvent_t start = nullptr; hipEvent_t stop = nullptr; };
// Small index arrays travel inside the kernel-argument segment (no upload, no staging buffer) when
// they fit; larger batches go through the pinned staging ring and are read through pointers.
constexpr int kInlineMaxReq = 256;
struct InlineMeta { int32_t v[3 * kInlineMaxReq + 2]; };

struct AppendArgs {
    const void* k_new; const void* v_new;   // [rows, H, D] bf16
    char* k_base; char* v_base;             // buffer bases of the layer
    int64_t S;                              // bytes between consecutive reqIds
    int64_t row_bytes;                      // H*D*P
    int64_t tok_stride;                     // bytes between consecutive tokens of the layer (H*D*P, or N*H*D*P when sliced)
    const int32_t* reqids; const int32_t* cu_q; const int32_t* kv_before;  // device, n / n+1 / n
    int n; int total_rows;
    int inline_meta;                        // 1: arrays are in InlineMeta as [reqids | kv_before | cu_q]
};
bool launch_append_kv(const AppendArgs& a, const InlineMeta* im, hipStream_t stream, LaunchEvents ev = {});

struct DecodeArgs {
    const void* q; void* o;                 // [n, Hq, D] bf16
    const char* k_base; const char* v_base; int64_t S;
    int Hq, H, D;
    int row_stride;                         // bytes between consecutive tokens of the layer
    // Split-K partition: the contexts of all requests, cut into 32-token tiles, form one global tile
    // sequence (request-major), cut into periods of `period` tiles; segment s owns tiles
    // [(s/8)*period + pre[s%8], (s/8)*period + pre[s%8 + 1]) - eight segment lengths that repeat, one per XCD
    // (segment s runs on XCD s % 8), so that XCDs which draw less bandwidth get shorter segments.  A segment
    // that crosses a request boundary produces one partial per request it touches.  The partial of
    // (segment s, request r) lives in slot s + r (strictly increasing along the sequence, so unique).
    const int32_t* reqids; const int32_t* kv_lens; const int32_t* cu_tiles;  // device: n, n, n+1
    int n; int total_tiles; int num_segs;
    int period; int pre[9];                 // pre[0] = 0 <= pre[1] <= ... <= pre[8] = period
    int max_slots;                          // most partials any one request has (picks the reduce kernel)
    float scale;
    float* part_o;   // [num_segs + n, Hq, D] un-normalised partial outputs
    float* part_ml;  // [num_segs + n, Hq, 2] running max (log2 domain) and partial sum
    int inline_meta; // 1: arrays are in InlineMeta as [reqids | kv_lens | cu_tiles]
    // Paged comparison variant only: k_base / v_base are block pools [num_blocks, block_tokens, H, D] and
    // block_table[req * table_stride + j] names the block holding tokens j*block_tokens .. of batch slot req.
    const int32_t* block_table; int table_stride; int block_tokens;
    // Fused append only: newest K/V rows [n, H, D] of the batch, to be stored at position kv_len - 1 (else null).
    const void* k_new; const void* v_new;
};
// Device address and size of the library-owned partials array of `device` (vattn_attn_decode_static).
constexpr size_t kDecodeScratchBytes = size_t{32} << 20;
bool decode_static_scratch(int device, void** ptr, size_t* bytes);
int decode_resident_workgroups(int Hq, int H, int D, int num_cus);  // workgroups one launch keeps resident
bool launch_decode_splitk(const DecodeArgs& a, const InlineMeta* im, hipStream_t stream, LaunchEvents ev = {});   // paged if a.block_table
bool launch_decode_reduce(const DecodeArgs& a, const InlineMeta* im, hipStream_t stream, LaunchEvents ev = {});

struct PrefillArgs {
    const void* q; void* o;                 // [sum q_len, Hq, D] bf16
    const char* k_base; const char* v_base; int64_t S;
    int Hq, H, D;
    int row_stride;                         // bytes between consecutive tokens of the layer
    const int32_t* reqids; const int32_t* cu_q; const int32_t* kv_lens;   // device
    const PrefillItem* items;               // device: 8 queues of items_per_xcd entries each
    int items_per_xcd; int n;
    int* queue_heads;                       // device: 8 counters, zero at launch: next slot of each XCD's queue (default kernel)
    int num_cus;
    int waves;                              // waves per workgroup (8 or 12); a work item is 32*waves rows
    // Paged comparison variant only (default kernel): k_base / v_base are block pools [num_blocks, block_tokens,
    // H, D]; block_table[req * table_stride + j] names the block with tokens j*block_tokens .. of batch slot req.
    const int32_t* block_table; int table_stride; int block_tokens;
    float scale;
    // Fused append only (default kernel, unsliced layout): K/V rows [sum q_len, H, D] of the query tokens, which the
    // kernel stores at positions kv_len - q_len .. kv_len - 1 and reads from here instead of from the cache (else null).
    const void* k_new; const void* v_new;
};
// 32 query rows per wave and `waves` = 8 or 12 waves per work item; one workgroup per CU.
// Measured on C3 / C5: 12 waves (three per SIMD) 1.18 / 1.22 PFLOP/s, 8 waves 1.13 / 1.19;
// 4 waves with two workgroups per CU 1.07 / 1.12; 6 waves at three per SIMD in two workgroups 0.97 / 1.00.
// Twelve waves need many work items: a 2048-token chunk (C4) runs 20 % slower with them than with eight.
bool launch_prefill(const PrefillArgs& a, hipStream_t stream, LaunchEvents ev = {});

}  // namespace vattn

struct vattn_ctx {
    vattn_config cfg{};
    vattn::KvMemory mem;
    vattn::MetaRing ring;
    vattn::KernelTimer timers[4];   // split-K decode, prefill, decode reduce, KV append
    bool timing = false;
    int decode_chunk = 0;
    int decode_oversub = 1;  // segments per resident workgroup slot
    float decode_xcd_weight[8] = {1.f, 0.9f, 1.f, 0.9f, 1.f, 0.9f, 1.f, 0.9f};   // relative segment length per XCD
    int num_cus = 0;
};
