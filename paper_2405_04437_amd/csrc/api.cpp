// C ABI of libvattn: argument checking, index marshalling and kernel launches.  All arithmetic of the
// attention path runs in the HIP kernels; this file only validates, packs index arrays into a pinned
// staging slot, uploads them on the caller's stream and launches.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "vattn_internal.h"

namespace vattn { const std::string& last_error_string(); }
using namespace vattn;

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool check_ctx_layer(vattn_ctx* ctx, int layer, const char* fn) {
    if (!ctx) { set_error(std::string(fn) + ": null context"); return false; }
    if (layer < 0 || layer >= ctx->cfg.num_layers) { set_error(std::string(fn) + ": layer out of range"); return false; }
    return true;
}

// A request may be attended to / appended to only if it is active and its context is fully backed.
bool check_request(vattn_ctx* ctx, int reqid, int64_t kv_len, const char* fn) {
    if (!ctx->mem.valid_reqid(reqid) || !ctx->mem.is_active(reqid)) {
        set_error(std::string(fn) + ": reqId " + std::to_string(reqid) + " out of range or not active");
        return false;
    }
    if (kv_len < 0 || kv_len > ctx->cfg.max_ctx || kv_len * ctx->mem.token_stride() > ctx->mem.mapped_committed(reqid) * ctx->mem.G()) {
        set_error(std::string(fn) + ": context length " + std::to_string(kv_len) + " of reqId " + std::to_string(reqid) +
                  " exceeds what step() has mapped");
        return false;
    }
    return true;
}

// Eq. 2 divides the scores by a positive constant; the kernels multiply by `scale` and rely on its sign (the
// prefill kernel takes row maxima before scaling).  Zero, negative, infinite or NaN values are refused.
bool check_scale(float scale, const char* fn) {
    if (std::isfinite(scale) && scale > 0.f) return true;
    set_error(std::string(fn) + ": scale must be finite and > 0");
    return false;
}

DecodePlan plan_decode(const vattn_ctx* ctx, const int64_t* kv_lens, int n) {
    const int resident = decode_resident_workgroups(ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, ctx->cfg.head_dim, ctx->num_cus);
    return make_decode_plan(kv_lens, n, ctx->decode_chunk, resident, ctx->decode_oversub, ctx->decode_xcd_weight);
}

size_t decode_part_o_bytes(const vattn_ctx* ctx, const DecodePlan& p, int n) {
    return align_up(static_cast<size_t>(p.num_segs + n) * ctx->cfg.num_q_heads * ctx->cfg.head_dim * 4, 256);
}
size_t decode_workspace_need(const vattn_ctx* ctx, const DecodePlan& p, int n) {
    return decode_part_o_bytes(ctx, p, n) + align_up(static_cast<size_t>(p.num_segs + n) * ctx->cfg.num_q_heads * 2 * 4, 256);
}

}  // namespace

extern "C" {

const char* vattn_last_error(void) { return last_error_string().c_str(); }

int vattn_init(const vattn_config* cfg, vattn_ctx** out) {
    if (!cfg || !out) { set_error("init: null argument"); return -1; }
    vattn_ctx* ctx = new (std::nothrow) vattn_ctx();
    if (!ctx) { set_error("init: out of host memory"); return -1; }
    ctx->cfg = *cfg;
    const VmmOps& ops = (cfg->flags & VATTN_FLAG_STATIC_BACKING) ? hip_static_ops() : hip_vmm_ops();
    if (!ctx->mem.init(*cfg, ops)) { delete ctx; return -1; }
    if (!hip_ok(hipDeviceGetAttribute(&ctx->num_cus, hipDeviceAttributeMultiprocessorCount, cfg->device), "hipDeviceGetAttribute") || ctx->num_cus <= 0) { delete ctx; return -1; }
    // Resolve the address of the library-owned decode scratch array on this device now, so that the allocation-free
    // entry point finds it ready even if its first call comes under graph capture (a failure is reported there).
    {
        void* p = nullptr; size_t b = 0;
        (void)decode_static_scratch(cfg->device, &p, &b);
    }
    *out = ctx;
    return 0;
}

int vattn_destroy(vattn_ctx* ctx) {
    if (!ctx) return 0;
    for (auto& t : ctx->timers) t.destroy();
    delete ctx;
    return 0;
}

int vattn_alloc_reqid(vattn_ctx* ctx) { return ctx ? ctx->mem.alloc_reqid() : (set_error("alloc_reqid: null context"), -1); }
int vattn_free_reqid(vattn_ctx* ctx, int reqid) { return ctx ? ctx->mem.free_reqid(reqid) : (set_error("free_reqid: null context"), -1); }
int vattn_step(vattn_ctx* ctx, const int64_t* seq_lens, int count) { return ctx ? ctx->mem.step(seq_lens, count) : (set_error("step: null context"), -1); }

void* vattn_kv_ptr(vattn_ctx* ctx, int layer, int which, int reqid) {
    if (!check_ctx_layer(ctx, layer, "kv_ptr")) return nullptr;
    if ((which != 0 && which != 1) || !ctx->mem.valid_reqid(reqid)) { set_error("kv_ptr: invalid argument"); return nullptr; }
    return ctx->mem.sub_tensor(layer, which, reqid);
}

int vattn_query(vattn_ctx* ctx, int reqid, int* active, int64_t* mapped, int64_t* va_offset) {
    if (!ctx || !ctx->mem.valid_reqid(reqid)) { set_error("query: invalid argument"); return -1; }
    if (active) *active = ctx->mem.is_active(reqid) ? 1 : 0;
    if (mapped) *mapped = ctx->mem.mapped(reqid);
    if (va_offset) *va_offset = static_cast<int64_t>(reqid) * ctx->mem.S();
    return 0;
}

int vattn_stats(vattn_ctx* ctx, int64_t* page_group_bytes, int64_t* S_bytes, int64_t* pool_total, int64_t* pool_free) {
    if (!ctx) { set_error("stats: null context"); return -1; }
    if (page_group_bytes) *page_group_bytes = ctx->mem.G();
    if (S_bytes) *S_bytes = ctx->mem.S();
    if (pool_total) *pool_total = ctx->mem.pool_total();
    if (pool_free) *pool_free = ctx->mem.pool_free();
    return 0;
}

int vattn_counters(vattn_ctx* ctx, int64_t* map_calls, int64_t* unmap_calls, double* map_us, double* unmap_us) {
    if (!ctx) { set_error("counters: null context"); return -1; }
    const KvMemory::Counters c = ctx->mem.counters();
    if (map_calls) *map_calls = c.map_calls;
    if (unmap_calls) *unmap_calls = c.unmap_calls;
    if (map_us) *map_us = c.map_us;
    if (unmap_us) *unmap_us = c.unmap_us;
    return 0;
}

int vattn_step_counters(vattn_ctx* ctx, int64_t* sync_map_calls, int64_t* background_map_calls, double* step_us,
                        double* background_us, double* wait_us) {
    if (!ctx) { set_error("step_counters: null context"); return -1; }
    const KvMemory::Counters c = ctx->mem.counters();
    if (sync_map_calls) *sync_map_calls = c.sync_map_calls;
    if (background_map_calls) *background_map_calls = c.background_map_calls;
    if (step_us) *step_us = c.step_us;
    if (background_us) *background_us = c.background_us;
    if (wait_us) *wait_us = c.wait_us;
    return 0;
}

int vattn_sync(vattn_ctx* ctx) {
    if (!ctx) { set_error("sync: null context"); return -1; }
    ctx->mem.sync();
    return 0;
}

int vattn_vmm_microbench(int device, int64_t bytes, int count, double* out_us) {
    return vmm_microbench(device, bytes, count, out_us) ? 0 : -1;
}

int vattn_stream_microbench(int device, int64_t bytes, double* out_gbs) {
    return stream_microbench(device, bytes, out_gbs) ? 0 : -1;
}

int vattn_mfma_microbench(int device, int normal_operands, int rounds, double* out) {
    if (!out) { set_error("mfma_microbench: null output"); return -1; }
    return mfma_microbench(device, normal_operands, rounds, &out[0], &out[1]) ? 0 : -1;
}

int vattn_append_kv(vattn_ctx* ctx, int layer, void* stream, const void* k_new, const void* v_new,
                    const int32_t* reqids, const int32_t* cu_q, const int64_t* kv_len_before, int n) {
    if (!check_ctx_layer(ctx, layer, "append_kv")) return -1;
    if (n < 0 || (n > 0 && (!k_new || !v_new || !reqids || !cu_q || !kv_len_before))) { set_error("append_kv: null argument"); return -1; }
    if (n == 0) return 0;
    if (cu_q[0] != 0) { set_error("append_kv: cu_q[0] must be 0"); return -1; }
    for (int r = 0; r < n; ++r) {
        const int64_t ql = static_cast<int64_t>(cu_q[r + 1]) - cu_q[r];
        if (ql < 0) { set_error("append_kv: cu_q must be non-decreasing"); return -1; }
        if (kv_len_before[r] < 0 || !check_request(ctx, reqids[r], kv_len_before[r] + ql, "append_kv")) return -1;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    LaunchEvents ev;
    if (ctx->timing && !ctx->timers[3].next(&ev.start, &ev.stop)) return -1;
    AppendArgs a{};
    a.k_new = k_new; a.v_new = v_new;
    a.k_base = ctx->mem.buffer_base(layer, 0); a.v_base = ctx->mem.buffer_base(layer, 1);
    a.S = ctx->mem.S(); a.row_bytes = ctx->mem.T(); a.tok_stride = ctx->mem.token_stride();
    a.n = n; a.total_rows = cu_q[n];
    if (n <= kInlineMaxReq) {
        InlineMeta im;
        for (int r = 0; r < n; ++r) { im.v[r] = reqids[r]; im.v[n + r] = static_cast<int32_t>(kv_len_before[r]); }
        for (int r = 0; r <= n; ++r) im.v[2 * n + r] = cu_q[r];
        a.inline_meta = 1;
        return launch_append_kv(a, &im, s, ev) ? 0 : -1;
    }
    const size_t off_kv = sizeof(int32_t) * n, off_cu = 2 * off_kv;
    const size_t bytes = off_cu + sizeof(int32_t) * (n + 1);
    char *h, *d;
    if (!ctx->ring.acquire(bytes, &h, &d)) return -1;
    std::memcpy(h, reqids, sizeof(int32_t) * n);
    for (int r = 0; r < n; ++r) reinterpret_cast<int32_t*>(h + off_kv)[r] = static_cast<int32_t>(kv_len_before[r]);
    std::memcpy(h + off_cu, cu_q, sizeof(int32_t) * (n + 1));
    if (!ctx->ring.commit(bytes, s)) return -1;
    a.reqids = reinterpret_cast<const int32_t*>(d);
    a.kv_before = reinterpret_cast<const int32_t*>(d + off_kv);
    a.cu_q = reinterpret_cast<const int32_t*>(d + off_cu);
    const bool ok = launch_append_kv(a, nullptr, s, ev);
    return ctx->ring.release(s) && ok ? 0 : -1;
}

int64_t vattn_decode_workspace_bytes(vattn_ctx* ctx, const int64_t* kv_lens, int n) {
    if (!ctx || n < 0 || (n > 0 && !kv_lens)) { set_error("decode_workspace_bytes: invalid argument"); return -1; }
    for (int i = 0; i < n; ++i)
        if (kv_lens[i] < 1) { set_error("decode_workspace_bytes: context lengths must be >= 1"); return -1; }
    DecodePlan p = plan_decode(ctx, kv_lens, n);
    if (ctx->decode_chunk == 0) {
        // In the balanced mode the segment count never exceeds the resident workgroup slots, whatever
        // the lengths: size for that bound so that the same workspace serves the batch as it grows.
        const int resident = decode_resident_workgroups(ctx->cfg.num_q_heads, ctx->cfg.num_kv_heads, ctx->cfg.head_dim, ctx->num_cus);
        p.num_segs = decode_plan_max_segs(resident, ctx->decode_oversub);
    }
    return static_cast<int64_t>(decode_workspace_need(ctx, p, n));
}

}  // extern "C"

namespace {

// Paged comparison variant: pools and block table instead of the context's virtual buffers.
struct PagedKv { const void* k_pool; const void* v_pool; int64_t num_blocks; int block_tokens; const int32_t* table; int table_stride; };
struct NewRows { const void* k_new; const void* v_new; };

// Shared by vattn_attn_decode and vattn_attn_decode_paged: split-K plan, index upload, the two launches.
int decode_common(vattn_ctx* ctx, int layer, void* stream, const void* q, void* o, const int32_t* reqids,
                  const int64_t* kv_lens, int n, float scale, void* workspace, size_t workspace_bytes, const PagedKv* paged,
                  const NewRows* fresh, const char* fn, bool no_alloc = false) {
    const DecodePlan plan = plan_decode(ctx, kv_lens, n);
    if (plan.total_tiles > INT32_MAX) { set_error(std::string(fn) + ": batch too large"); return -1; }
    const bool inl = n <= kInlineMaxReq && !paged;
    // The allocation-free entry point must stay clear of the staging ring (which grows with hipMalloc) and of
    // the timers (which create events): its index arrays travel in the kernel arguments only.
    if (no_alloc && !inl) { set_error(std::string(fn) + ": at most " + std::to_string(kInlineMaxReq) + " requests per call"); return -1; }
    InlineMeta im;
    const size_t off_kv = sizeof(int32_t) * n, off_cu = off_kv * 2;
    const size_t off_tab = align_up(off_cu + sizeof(int32_t) * (n + 1), 16);
    const size_t tab_bytes = paged ? sizeof(int32_t) * static_cast<size_t>(n) * paged->table_stride : 0;
    const size_t bytes = paged ? off_tab + tab_bytes : off_cu + sizeof(int32_t) * (n + 1);
    char *h = nullptr, *d = nullptr;
    if (!inl && !ctx->ring.acquire(bytes, &h, &d)) return -1;
    int32_t* h_req = inl ? im.v : reinterpret_cast<int32_t*>(h);
    int32_t* h_kv = inl ? im.v + n : reinterpret_cast<int32_t*>(h + off_kv);
    int32_t* h_cu = inl ? im.v + 2 * n : reinterpret_cast<int32_t*>(h + off_cu);
    int64_t total = 0;
    for (int r = 0; r < n; ++r) {
        h_req[r] = reqids ? reqids[r] : 0;
        h_kv[r] = static_cast<int32_t>(kv_lens[r]);
        h_cu[r] = static_cast<int32_t>(total);
        total += (kv_lens[r] + 31) / 32;
    }
    h_cu[n] = static_cast<int32_t>(total);
    if (paged) std::memcpy(h + off_tab, paged->table, tab_bytes);
    const int Hq = ctx->cfg.num_q_heads, D = ctx->cfg.head_dim;
    const size_t part_o_bytes = decode_part_o_bytes(ctx, plan, n);
    const size_t need = decode_workspace_need(ctx, plan, n);
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) { set_error(std::string(fn) + ": workspace must be 256-byte aligned"); return -1; }
    if (workspace_bytes < need) { set_error(std::string(fn) + ": workspace too small (" + std::to_string(workspace_bytes) + " < " + std::to_string(need) + ")"); return -1; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!inl && !ctx->ring.commit(bytes, s)) return -1;

    DecodeArgs a{};
    a.q = q; a.o = o;
    if (paged) {
        a.k_base = static_cast<const char*>(paged->k_pool); a.v_base = static_cast<const char*>(paged->v_pool); a.S = 0;
        a.row_stride = static_cast<int>(ctx->mem.T());
        a.block_table = reinterpret_cast<const int32_t*>(d + off_tab); a.table_stride = paged->table_stride; a.block_tokens = paged->block_tokens;
    } else {
        a.k_base = ctx->mem.buffer_base(layer, 0); a.v_base = ctx->mem.buffer_base(layer, 1); a.S = ctx->mem.S();
        a.row_stride = static_cast<int>(ctx->mem.token_stride());
    }
    a.Hq = Hq; a.H = ctx->cfg.num_kv_heads; a.D = D;
    if (fresh) { a.k_new = fresh->k_new; a.v_new = fresh->v_new; }
    a.inline_meta = inl ? 1 : 0;
    a.reqids = reinterpret_cast<const int32_t*>(d);
    a.kv_lens = reinterpret_cast<const int32_t*>(d + off_kv);
    a.cu_tiles = reinterpret_cast<const int32_t*>(d + off_cu);
    a.n = n; a.total_tiles = static_cast<int>(total); a.num_segs = plan.num_segs; a.scale = scale;
    a.period = plan.period;
    for (int x = 0; x < 9; ++x) a.pre[x] = plan.pre[x];
    {
        int64_t most = 1;
        for (int r = 0; r < n; ++r)
            most = std::max<int64_t>(most, decode_plan_segment_of(plan, h_cu[r + 1] - 1) - decode_plan_segment_of(plan, h_cu[r]) + 1);
        a.max_slots = static_cast<int>(most);
    }
    a.part_o = static_cast<float*>(workspace);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + part_o_bytes);
    const InlineMeta* imp = inl ? &im : nullptr;
    LaunchEvents ev_split, ev_reduce;
    if (ctx->timing && !no_alloc && (!ctx->timers[0].next(&ev_split.start, &ev_split.stop) || !ctx->timers[2].next(&ev_reduce.start, &ev_reduce.stop))) {
        if (!inl) (void)ctx->ring.release(s);
        return -1;
    }
    const bool ok = launch_decode_splitk(a, imp, s, ev_split) && launch_decode_reduce(a, imp, s, ev_reduce);
    if (!inl && !ctx->ring.release(s)) return -1;   // the staging slot stays taken until both kernels have read it
    return ok ? 0 : -1;
}

}  // namespace

extern "C" {

int vattn_attn_decode(vattn_ctx* ctx, int layer, void* stream, const void* q, void* o, const int32_t* reqids,
                      const int64_t* kv_lens, int n, float scale, void* workspace, size_t workspace_bytes) {
    if (!check_scale(scale, "attn_decode")) return -1;
    if (!check_ctx_layer(ctx, layer, "attn_decode")) return -1;
    if (n < 0 || (n > 0 && (!q || !o || !reqids || !kv_lens || !workspace))) { set_error("attn_decode: null argument"); return -1; }
    if (n == 0) return 0;
    for (int r = 0; r < n; ++r) {
        if (kv_lens[r] < 1) { set_error("attn_decode: context length must be >= 1"); return -1; }
        if (!check_request(ctx, reqids[r], kv_lens[r], "attn_decode")) return -1;
    }
    return decode_common(ctx, layer, stream, q, o, reqids, kv_lens, n, scale, workspace, workspace_bytes, nullptr, nullptr, "attn_decode");
}

int vattn_attn_decode_static(vattn_ctx* ctx, int layer, void* stream, const void* q, void* o, const int32_t* reqids,
                             const int64_t* kv_lens, int n, float scale) {
    if (!check_scale(scale, "attn_decode_static")) return -1;
    if (!check_ctx_layer(ctx, layer, "attn_decode_static")) return -1;
    if (n < 0 || (n > 0 && (!q || !o || !reqids || !kv_lens))) { set_error("attn_decode_static: null argument"); return -1; }
    if (n == 0) return 0;
    for (int r = 0; r < n; ++r) {
        if (kv_lens[r] < 1) { set_error("attn_decode_static: context length must be >= 1"); return -1; }
        if (!check_request(ctx, reqids[r], kv_lens[r], "attn_decode_static")) return -1;
    }
    void* scratch_ptr = nullptr;
    size_t scratch_bytes = 0;
    if (!decode_static_scratch(ctx->cfg.device, &scratch_ptr, &scratch_bytes)) return -1;
    const size_t need = decode_workspace_need(ctx, plan_decode(ctx, kv_lens, n), n);
    if (need > scratch_bytes) {
        set_error("attn_decode_static: this batch needs " + std::to_string(need) + " bytes of split-K partials, the library-owned array holds " +
                  std::to_string(scratch_bytes) + "; use vattn_attn_decode with a caller-owned workspace");
        return -1;
    }
    return decode_common(ctx, layer, stream, q, o, reqids, kv_lens, n, scale, scratch_ptr, scratch_bytes, nullptr, nullptr, "attn_decode_static", true);
}

int vattn_attn_decode_append(vattn_ctx* ctx, int layer, void* stream, const void* q, const void* k_new, const void* v_new, void* o,
                             const int32_t* reqids, const int64_t* kv_lens, int n, float scale, void* workspace, size_t workspace_bytes) {
    if (!check_scale(scale, "attn_decode_append")) return -1;
    if (!check_ctx_layer(ctx, layer, "attn_decode_append")) return -1;
    if (n < 0 || (n > 0 && (!q || !k_new || !v_new || !o || !reqids || !kv_lens || !workspace))) { set_error("attn_decode_append: null argument"); return -1; }
    if (n == 0) return 0;
    for (int r = 0; r < n; ++r) {
        if (kv_lens[r] < 1) { set_error("attn_decode_append: context length must be >= 1"); return -1; }
        if (!check_request(ctx, reqids[r], kv_lens[r], "attn_decode_append")) return -1;
        for (int p = 0; p < r; ++p)
            if (reqids[p] == reqids[r]) { set_error("attn_decode_append: a reqId appears twice in the batch"); return -1; }
    }
    const NewRows fresh{k_new, v_new};
    return decode_common(ctx, layer, stream, q, o, reqids, kv_lens, n, scale, workspace, workspace_bytes, nullptr, &fresh, "attn_decode_append");
}

int vattn_attn_decode_paged(vattn_ctx* ctx, void* stream, const void* q, void* o, const void* k_pool, const void* v_pool,
                            int64_t num_blocks, int block_tokens, const int32_t* block_table, int max_blocks_per_req,
                            const int64_t* kv_lens, int n, float scale, void* workspace, size_t workspace_bytes) {
    if (!check_scale(scale, "attn_decode_paged")) return -1;
    if (!ctx) { set_error("attn_decode_paged: null context"); return -1; }
    if (n < 0 || (n > 0 && (!q || !o || !k_pool || !v_pool || !block_table || !kv_lens || !workspace))) { set_error("attn_decode_paged: null argument"); return -1; }
    if (n == 0) return 0;
    if (block_tokens < 32 || block_tokens % 32 != 0) { set_error("attn_decode_paged: block_tokens must be a positive multiple of 32"); return -1; }
    if (num_blocks <= 0 || num_blocks > INT32_MAX || max_blocks_per_req <= 0) { set_error("attn_decode_paged: invalid pool or table size"); return -1; }
    for (int r = 0; r < n; ++r) {
        if (kv_lens[r] < 1 || kv_lens[r] > static_cast<int64_t>(max_blocks_per_req) * block_tokens) {
            set_error("attn_decode_paged: context length of slot " + std::to_string(r) + " does not fit its block-table row");
            return -1;
        }
        const int64_t used = (kv_lens[r] + block_tokens - 1) / block_tokens;
        for (int64_t j = 0; j < used; ++j) {
            const int32_t b = block_table[static_cast<int64_t>(r) * max_blocks_per_req + j];
            if (b < 0 || b >= num_blocks) { set_error("attn_decode_paged: block index out of range in slot " + std::to_string(r)); return -1; }
        }
    }
    const PagedKv pk{k_pool, v_pool, num_blocks, block_tokens, block_table, max_blocks_per_req};
    return decode_common(ctx, 0, stream, q, o, nullptr, kv_lens, n, scale, workspace, workspace_bytes, &pk, nullptr, "attn_decode_paged");
}

}  // extern "C"

namespace {

// Shared by vattn_attn_prefill and vattn_attn_prefill_paged: work queues per XCD, index upload, launch.
// The callers have validated the requests.
int prefill_common(vattn_ctx* ctx, int layer, void* stream, const void* q, void* o, const int32_t* reqids,
                   const int32_t* cu_q, const int64_t* kv_lens, int n, float scale, const PagedKv* paged, const NewRows* fresh = nullptr) {
    const int H = ctx->cfg.num_kv_heads, Hq = ctx->cfg.num_q_heads, D = ctx->cfg.head_dim;
    const PrefillQueues queues = make_prefill_queues(reqids, cu_q, kv_lens, n, Hq, H, ctx->num_cus);
    const int waves = queues.waves;
    const size_t per_xcd = static_cast<size_t>(queues.per_xcd);
    if (per_xcd == 0) return 0;
    const size_t off_cu = sizeof(int32_t) * n;
    const size_t off_kv = off_cu + sizeof(int32_t) * (n + 1);
    const size_t off_items = align_up(off_kv + sizeof(int32_t) * n, 16);
    const size_t off_tab = align_up(off_items + sizeof(PrefillItem) * per_xcd * 8, 16);
    const size_t tab_bytes = paged ? sizeof(int32_t) * static_cast<size_t>(n) * paged->table_stride : 0;
    const size_t off_ctr = align_up(off_tab + tab_bytes, 16);   // queue counters, uploaded as zeros with the rest
    const size_t bytes = off_ctr + 8 * sizeof(int32_t);
    char *h, *d;
    if (!ctx->ring.acquire(bytes, &h, &d)) return -1;
    std::memset(h + off_ctr, 0, 8 * sizeof(int32_t));
    if (reqids) std::memcpy(h, reqids, sizeof(int32_t) * n);
    else std::memset(h, 0, sizeof(int32_t) * n);
    if (paged) std::memcpy(h + off_tab, paged->table, tab_bytes);
    std::memcpy(h + off_cu, cu_q, sizeof(int32_t) * (n + 1));
    int32_t* h_kv = reinterpret_cast<int32_t*>(h + off_kv);
    for (int r = 0; r < n; ++r) h_kv[r] = static_cast<int32_t>(kv_lens[r]);
    std::memcpy(h + off_items, queues.items.data(), sizeof(PrefillItem) * per_xcd * 8);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!ctx->ring.commit(bytes, s)) return -1;

    PrefillArgs a{};
    a.q = q; a.o = o;
    if (paged) {
        a.k_base = static_cast<const char*>(paged->k_pool); a.v_base = static_cast<const char*>(paged->v_pool); a.S = 0;
        a.row_stride = static_cast<int>(ctx->mem.T());
        a.block_table = reinterpret_cast<const int32_t*>(d + off_tab); a.table_stride = paged->table_stride; a.block_tokens = paged->block_tokens;
    } else {
        a.k_base = ctx->mem.buffer_base(layer, 0); a.v_base = ctx->mem.buffer_base(layer, 1); a.S = ctx->mem.S();
        a.row_stride = static_cast<int>(ctx->mem.token_stride());
    }
    a.Hq = Hq; a.H = H; a.D = D;
    a.reqids = reinterpret_cast<const int32_t*>(d);
    a.cu_q = reinterpret_cast<const int32_t*>(d + off_cu);
    a.kv_lens = reinterpret_cast<const int32_t*>(d + off_kv);
    a.items = reinterpret_cast<const PrefillItem*>(d + off_items);
    a.items_per_xcd = static_cast<int>(per_xcd); a.n = n; a.scale = scale; a.waves = waves;
    a.queue_heads = reinterpret_cast<int*>(d + off_ctr); a.num_cus = ctx->num_cus;
    if (fresh) { a.k_new = fresh->k_new; a.v_new = fresh->v_new; }
    LaunchEvents ev;
    if (ctx->timing && !ctx->timers[1].next(&ev.start, &ev.stop)) { (void)ctx->ring.release(s); return -1; }
    const bool ok = launch_prefill(a, s, ev);
    return ctx->ring.release(s) && ok ? 0 : -1;   // the slot (index arrays, work queues, queue counters) stays taken until the kernel ends
}

}  // namespace

extern "C" {

int vattn_attn_prefill(vattn_ctx* ctx, int layer, void* stream, const void* q, void* o, const int32_t* reqids,
                       const int32_t* cu_q, const int64_t* kv_lens, int n, float scale) {
    if (!check_scale(scale, "attn_prefill")) return -1;
    if (!check_ctx_layer(ctx, layer, "attn_prefill")) return -1;
    if (n < 0 || (n > 0 && (!q || !o || !reqids || !cu_q || !kv_lens))) { set_error("attn_prefill: null argument"); return -1; }
    if (n == 0) return 0;
    if (cu_q[0] != 0) { set_error("attn_prefill: cu_q[0] must be 0"); return -1; }
    for (int r = 0; r < n; ++r) {
        const int64_t ql = static_cast<int64_t>(cu_q[r + 1]) - cu_q[r];
        if (ql < 0) { set_error("attn_prefill: cu_q must be non-decreasing"); return -1; }
        if (kv_lens[r] < ql) { set_error("attn_prefill: kv_len < q_len for batch slot " + std::to_string(r)); return -1; }
        if (ql > 0 && !check_request(ctx, reqids[r], kv_lens[r], "attn_prefill")) return -1;
    }
    return prefill_common(ctx, layer, stream, q, o, reqids, cu_q, kv_lens, n, scale, nullptr);
}

int vattn_attn_prefill_append(vattn_ctx* ctx, int layer, void* stream, const void* q, const void* k_new, const void* v_new, void* o,
                              const int32_t* reqids, const int32_t* cu_q, const int64_t* kv_lens, int n, float scale) {
    if (!check_scale(scale, "attn_prefill_append")) return -1;
    if (!check_ctx_layer(ctx, layer, "attn_prefill_append")) return -1;
    if (n < 0 || (n > 0 && (!q || !k_new || !v_new || !o || !reqids || !cu_q || !kv_lens))) { set_error("attn_prefill_append: null argument"); return -1; }
    if (n == 0) return 0;
    if (cu_q[0] != 0) { set_error("attn_prefill_append: cu_q[0] must be 0"); return -1; }
    for (int r = 0; r < n; ++r) {
        const int64_t ql = static_cast<int64_t>(cu_q[r + 1]) - cu_q[r];
        if (ql < 0) { set_error("attn_prefill_append: cu_q must be non-decreasing"); return -1; }
        if (kv_lens[r] < ql) { set_error("attn_prefill_append: kv_len < q_len for batch slot " + std::to_string(r)); return -1; }
        if (ql > 0 && !check_request(ctx, reqids[r], kv_lens[r], "attn_prefill_append")) return -1;
        for (int p = 0; ql > 0 && p < r; ++p)
            if (reqids[p] == reqids[r] && cu_q[p + 1] > cu_q[p]) { set_error("attn_prefill_append: a reqId appears twice in the batch"); return -1; }
    }
    const NewRows fresh{k_new, v_new};
    return prefill_common(ctx, layer, stream, q, o, reqids, cu_q, kv_lens, n, scale, nullptr, &fresh);
}

int vattn_attn_prefill_paged(vattn_ctx* ctx, void* stream, const void* q, void* o, const void* k_pool, const void* v_pool,
                             int64_t num_blocks, int block_tokens, const int32_t* block_table, int max_blocks_per_req,
                             const int32_t* cu_q, const int64_t* kv_lens, int n, float scale) {
    if (!check_scale(scale, "attn_prefill_paged")) return -1;
    if (!ctx) { set_error("attn_prefill_paged: null context"); return -1; }
    if (n < 0 || (n > 0 && (!q || !o || !k_pool || !v_pool || !block_table || !cu_q || !kv_lens))) { set_error("attn_prefill_paged: null argument"); return -1; }
    if (n == 0) return 0;
    if (cu_q[0] != 0) { set_error("attn_prefill_paged: cu_q[0] must be 0"); return -1; }
    if (block_tokens < 64 || block_tokens % 64 != 0) { set_error("attn_prefill_paged: block_tokens must be a positive multiple of 64"); return -1; }
    if (num_blocks <= 0 || num_blocks > INT32_MAX || max_blocks_per_req <= 0) { set_error("attn_prefill_paged: invalid pool or table size"); return -1; }
    for (int r = 0; r < n; ++r) {
        const int64_t ql = static_cast<int64_t>(cu_q[r + 1]) - cu_q[r];
        if (ql < 0) { set_error("attn_prefill_paged: cu_q must be non-decreasing"); return -1; }
        if (kv_lens[r] < ql || kv_lens[r] > static_cast<int64_t>(max_blocks_per_req) * block_tokens) {
            set_error("attn_prefill_paged: context length of slot " + std::to_string(r) + " is below q_len or does not fit its block-table row");
            return -1;
        }
        const int64_t used = (kv_lens[r] + block_tokens - 1) / block_tokens;
        for (int64_t j = 0; j < used; ++j) {
            const int32_t b = block_table[static_cast<int64_t>(r) * max_blocks_per_req + j];
            if (b < 0 || b >= num_blocks) { set_error("attn_prefill_paged: block index out of range in slot " + std::to_string(r)); return -1; }
        }
    }
    const PagedKv pk{k_pool, v_pool, num_blocks, block_tokens, block_table, max_blocks_per_req};
    return prefill_common(ctx, 0, stream, q, o, nullptr, cu_q, kv_lens, n, scale, &pk);
}

int vattn_set_timing(vattn_ctx* ctx, int enabled) {
    if (!ctx) { set_error("set_timing: null context"); return -1; }
    ctx->timing = enabled != 0;
    return 0;
}

int vattn_kernel_time(vattn_ctx* ctx, int which, double* total_ms, int64_t* launches) {
    if (!ctx || which < 0 || which > 3) { set_error("kernel_time: invalid argument"); return -1; }
    return ctx->timers[which].collect(total_ms, launches) ? 0 : -1;
}

int vattn_set_decode_chunk(vattn_ctx* ctx, int tokens) {
    if (!ctx || tokens < 0 || tokens % 32 != 0) { set_error("set_decode_chunk: tokens must be a non-negative multiple of 32"); return -1; }
    ctx->decode_chunk = tokens;
    return 0;
}

int vattn_set_decode_tuning(vattn_ctx* ctx, int segments_per_slot) {
    if (!ctx || segments_per_slot < 1 || segments_per_slot > 64) {
        set_error("set_decode_tuning: segments_per_slot must be in [1,64]");
        return -1;
    }
    ctx->decode_oversub = segments_per_slot;
    return 0;
}

int vattn_set_decode_xcd_weights(vattn_ctx* ctx, const float* weights) {
    if (!ctx) { set_error("set_decode_xcd_weights: null context"); return -1; }
    static const float kDefault[8] = {1.f, 0.9f, 1.f, 0.9f, 1.f, 0.9f, 1.f, 0.9f};
    const float* w = weights ? weights : kDefault;
    for (int x = 0; x < 8; ++x)
        if (!(w[x] >= 0.25f && w[x] <= 4.f)) { set_error("set_decode_xcd_weights: weights must lie in [0.25, 4]"); return -1; }
    for (int x = 0; x < 8; ++x) ctx->decode_xcd_weight[x] = w[x];
    return 0;
}

}  // extern "C"
