// KV-cache memory manager on the HIP virtual-memory API.
//
// Design (Sec. 5 of the paper, re-expressed for HIP): virtual address space is reserved once for
// the largest batch and context (hipMemAddressReserve), physical page-groups are created up front
// (hipMemCreate) but mapped (hipMemMap + hipMemSetAccess) only when step() sees that a request's
// context has outgrown what is backed.  One physical handle per page-group: HIP rejects mapping a
// handle at a non-zero offset, so a page-group is the unit of both creation and mapping.
#include <chrono>
#include <thread>

#include "vattn_internal.h"

namespace vattn {

namespace {
thread_local std::string g_error;
double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
}  // namespace

void set_error(const std::string& msg) { g_error = msg; }
const std::string& last_error_string() { return g_error; }

bool hip_ok(hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    (void)hipGetLastError();  // clear the sticky error so later calls are not blamed for it
    return false;
}

bool KvMemory::init(const vattn_config& c) {
    if (c.num_layers <= 0 || c.max_batch <= 0 || c.max_ctx <= 0 || c.num_kv_heads <= 0 ||
        c.num_q_heads <= 0 || c.num_q_heads % c.num_kv_heads != 0) {
        set_error("init: N, B, L, H must be positive and Hq a multiple of H");
        return false;
    }
    if (c.head_dim != 64 && c.head_dim != 128) { set_error("init: head_dim must be 64 or 128"); return false; }
    if (c.elem_bytes != 2) { set_error("init: only 2-byte (bf16) elements are supported"); return false; }
    if (c.flags != VATTN_POLICY_SYNC_UNMAP && c.flags != VATTN_POLICY_DEFERRED) { set_error("init: unknown policy flag"); return false; }
    device_ = c.device;
    if (!hip_ok(hipSetDevice(device_), "hipSetDevice")) return false;
    int vmm = 0;
    if (!hip_ok(hipDeviceGetAttribute(&vmm, hipDeviceAttributeVirtualMemoryManagementSupported, device_), "hipDeviceGetAttribute")) return false;
    if (!vmm) { set_error("init: device does not support virtual memory management"); return false; }

    hipMemAllocationProp prop{};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device_;
    size_t gran = 0;
    if (!hip_ok(hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum), "hipMemGetAllocationGranularity")) return false;
    if (gran == 0) { set_error("init: zero allocation granularity"); return false; }
    int64_t G = c.page_group_bytes == 0 ? (int64_t{2} << 20) : c.page_group_bytes;
    if (c.page_group_bytes == 0) G = (G + static_cast<int64_t>(gran) - 1) / static_cast<int64_t>(gran) * static_cast<int64_t>(gran);
    if (G <= 0 || G % static_cast<int64_t>(gran) != 0) {
        set_error("init: page_group_bytes must be a positive multiple of the allocation granularity (" + std::to_string(gran) + ")");
        return false;
    }
    N_ = c.num_layers; B_ = c.max_batch; L_ = c.max_ctx; policy_ = c.flags; G_ = G;
    T_ = static_cast<int64_t>(c.num_kv_heads) * c.head_dim * c.elem_bytes;
    S_ = (L_ * T_ + G_ - 1) / G_ * G_;
    if (S_ >= (int64_t{1} << 31)) { set_error("init: one request's sub-tensor (L*H*D*P) must stay below 2 GiB (32-bit buffer offsets in the kernels)"); return false; }
    pool_total_ = c.phys_budget_bytes / G_;
    if (pool_total_ < 0) { set_error("init: negative physical budget"); return false; }

    access_.location.type = hipMemLocationTypeDevice;
    access_.location.id = device_;
    access_.flags = hipMemAccessFlagsProtReadWrite;

    const size_t buf_bytes = static_cast<size_t>(B_) * static_cast<size_t>(S_);
    base_.assign(static_cast<size_t>(2) * N_, nullptr);
    for (size_t b = 0; b < base_.size(); ++b) {
        void* p = nullptr;
        if (!hip_ok(hipMemAddressReserve(&p, buf_bytes, static_cast<size_t>(G_), nullptr, 0), "hipMemAddressReserve")) return false;
        base_[b] = static_cast<char*>(p);
    }
    free_handles_.reserve(static_cast<size_t>(pool_total_));
    for (int64_t i = 0; i < pool_total_; ++i) {
        hipMemGenericAllocationHandle_t h;
        if (!hip_ok(hipMemCreate(&h, static_cast<size_t>(G_), &prop, 0), "hipMemCreate (physical pool)")) return false;
        free_handles_.push_back(h);
    }
    held_.assign(static_cast<size_t>(B_), {});
    active_.assign(static_cast<size_t>(B_), 0);
    mapped_.assign(static_cast<size_t>(B_), 0);
    return true;
}

KvMemory::~KvMemory() {
    if (base_.empty()) return;
    (void)hipSetDevice(device_);
    (void)hipDeviceSynchronize();
    for (int r = 0; r < B_; ++r) unmap_rows(r, 0);
    for (auto h : free_handles_) (void)hipMemRelease(h);
    const size_t buf_bytes = static_cast<size_t>(B_) * static_cast<size_t>(S_);
    for (char* p : base_) if (p) (void)hipMemAddressFree(p, buf_bytes);
}

int KvMemory::alloc_reqid() {
    int best = -1;
    for (int r = 0; r < B_; ++r) {
        if (active_[r]) continue;
        if (best < 0) { best = r; if (policy_ == VATTN_POLICY_SYNC_UNMAP) break; continue; }
        if (mapped_[r] > mapped_[best]) best = r;  // most pages still mapped; ties keep the lowest id
    }
    if (best < 0) { set_error("alloc_reqid: all reqIds are in use"); return -1; }
    active_[best] = 1;
    return best;
}

int KvMemory::free_reqid(int r) {
    if (!valid_reqid(r) || !active_[r]) { set_error("free_reqid: reqId out of range or not active"); return -1; }
    active_[r] = 0;
    if (policy_ == VATTN_POLICY_SYNC_UNMAP) unmap_rows(r, 0);
    return 0;
}

bool KvMemory::map_rows(int r, int64_t from, int64_t to) {
    const size_t nb = base_.size();
    auto& held = held_[r];
    const double t0 = now_us();
    for (int64_t k = from; k < to; ++k) {
        for (size_t b = 0; b < nb; ++b) {
            hipMemGenericAllocationHandle_t h = free_handles_.back();
            char* va = base_[b] + static_cast<int64_t>(r) * S_ + k * G_;
            if (!hip_ok(hipMemMap(va, static_cast<size_t>(G_), 0, h, 0), "hipMemMap")) {
                // undo the partial row and everything mapped by this call
                for (size_t u = 0; u < b; ++u) {
                    (void)hipMemUnmap(base_[u] + static_cast<int64_t>(r) * S_ + k * G_, static_cast<size_t>(G_));
                    free_handles_.push_back(held.back()); held.pop_back();
                }
                mapped_[r] = k; unmap_rows(r, from);
                return false;
            }
            free_handles_.pop_back();
            held.push_back(h);
            ++map_calls;
        }
        mapped_[r] = k + 1;
    }
    // One access call per buffer covers the whole newly mapped, contiguous range.
    for (size_t b = 0; b < nb; ++b) {
        char* va = base_[b] + static_cast<int64_t>(r) * S_ + from * G_;
        if (!hip_ok(hipMemSetAccess(va, static_cast<size_t>((to - from) * G_), &access_, 1), "hipMemSetAccess")) {
            unmap_rows(r, from);
            return false;
        }
    }
    map_us += now_us() - t0;
    return true;
}

void KvMemory::unmap_rows(int r, int64_t keep) {
    const size_t nb = base_.size();
    auto& held = held_[r];
    const double t0 = now_us();
    for (int64_t k = mapped_[r] - 1; k >= keep; --k) {
        for (size_t b = nb; b-- > 0;) {
            (void)hipMemUnmap(base_[b] + static_cast<int64_t>(r) * S_ + k * G_, static_cast<size_t>(G_));
            free_handles_.push_back(held.back());
            held.pop_back();
            ++unmap_calls;
        }
    }
    if (mapped_[r] > keep) mapped_[r] = keep;
    unmap_us += now_us() - t0;
}

int KvMemory::step(const int64_t* seq_lens, int count) {
    if (!seq_lens || count != B_) { set_error("step: seq_lens must have exactly B entries"); return -1; }
    std::vector<int64_t> want(static_cast<size_t>(B_), 0);
    int64_t demand_rows = 0, reclaimable_rows = 0;
    for (int r = 0; r < B_; ++r) {
        const int64_t n = seq_lens[r];
        if (n < 0 || n > L_) { set_error("step: sequence length out of range for reqId " + std::to_string(r)); return -1; }
        if (!active_[r]) {
            if (n != 0) { set_error("step: non-zero length for inactive reqId " + std::to_string(r)); return -1; }
            reclaimable_rows += mapped_[r];
            continue;
        }
        const int64_t need = (n * T_ + G_ - 1) / G_;  // (s + t - 1) / t
        want[r] = need > mapped_[r] ? need : mapped_[r];
        demand_rows += want[r] - mapped_[r];
    }
    const int64_t per_row = static_cast<int64_t>(base_.size());
    const int64_t demand = demand_rows * per_row;
    if (demand > pool_free() + reclaimable_rows * per_row) {
        set_error("step: physical pool exhausted (demand " + std::to_string(demand) + " page-groups, free " + std::to_string(pool_free()) + ")");
        return -1;
    }
    if (demand > pool_free()) {  // deferred policy: take pages back from inactive ids, lowest id first
        for (int r = 0; r < B_ && pool_free() < demand; ++r) {
            if (active_[r]) continue;
            while (mapped_[r] > 0 && pool_free() < demand) unmap_rows(r, mapped_[r] - 1);
        }
    }
    for (int r = 0; r < B_; ++r) {
        if (!active_[r] || want[r] <= mapped_[r]) continue;
        if (!map_rows(r, mapped_[r], want[r])) return -1;
    }
    return 0;
}

// ---------------------------------------------------------------------------------------------

MetaRing::~MetaRing() {
    for (int i = 0; i < kSlots; ++i) if (ev_[i]) (void)hipEventDestroy(ev_[i]);
    if (host_) (void)hipHostFree(host_);
    if (dev_) (void)hipFree(dev_);
}

bool MetaRing::grow(size_t bytes) {
    if (!hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize")) return false;
    if (host_) { (void)hipHostFree(host_); host_ = nullptr; }
    if (dev_) { (void)hipFree(dev_); dev_ = nullptr; }
    size_t sz = 64 * 1024;
    while (sz < bytes) sz *= 2;
    if (!hip_ok(hipHostMalloc(reinterpret_cast<void**>(&host_), sz * kSlots, hipHostMallocDefault), "hipHostMalloc")) return false;
    if (!hip_ok(hipMalloc(reinterpret_cast<void**>(&dev_), sz * kSlots), "hipMalloc (index staging)")) return false;
    slot_bytes_ = sz;
    for (int i = 0; i < kSlots; ++i) {
        pending_[i] = false;
        if (!ev_[i] && !hip_ok(hipEventCreateWithFlags(&ev_[i], hipEventDisableTiming), "hipEventCreate")) return false;
    }
    return true;
}

bool MetaRing::acquire(size_t bytes, char** host, char** dev) {
    if (bytes > slot_bytes_ && !grow(bytes)) return false;
    cur_ = (cur_ + 1) % kSlots;
    if (pending_[cur_]) {
        if (!hip_ok(hipEventSynchronize(ev_[cur_]), "hipEventSynchronize")) return false;
        pending_[cur_] = false;
    }
    *host = host_ + static_cast<size_t>(cur_) * slot_bytes_;
    *dev = dev_ + static_cast<size_t>(cur_) * slot_bytes_;
    return true;
}

bool MetaRing::commit(size_t bytes, hipStream_t stream) {
    char* h = host_ + static_cast<size_t>(cur_) * slot_bytes_;
    char* d = dev_ + static_cast<size_t>(cur_) * slot_bytes_;
    if (!hip_ok(hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, stream), "hipMemcpyAsync (index upload)")) return false;
    if (!hip_ok(hipEventRecord(ev_[cur_], stream), "hipEventRecord")) return false;
    pending_[cur_] = true;
    return true;
}

// ---------------------------------------------------------------------------------------------

bool KernelTimer::next(hipEvent_t* start, hipEvent_t* stop) {
    Pair p{};
    if (!spare.empty()) { p = spare.back(); spare.pop_back(); }
    else {
        if (!hip_ok(hipEventCreate(&p.a), "hipEventCreate")) return false;
        if (!hip_ok(hipEventCreate(&p.b), "hipEventCreate")) return false;
    }
    open.push_back(p);
    *start = p.a; *stop = p.b;
    return true;
}
bool KernelTimer::collect(double* total_ms, int64_t* launches) {
    double t = 0;
    for (auto& p : open) {
        if (!hip_ok(hipEventSynchronize(p.b), "hipEventSynchronize")) return false;
        float ms = 0;
        if (!hip_ok(hipEventElapsedTime(&ms, p.a, p.b), "hipEventElapsedTime")) return false;
        t += ms;
        spare.push_back(p);
    }
    if (total_ms) *total_ms = t;
    if (launches) *launches = static_cast<int64_t>(open.size());
    open.clear();
    return true;
}
void KernelTimer::destroy() {
    for (auto& p : open) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    for (auto& p : spare) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    open.clear(); spare.clear();
}

}  // namespace vattn
