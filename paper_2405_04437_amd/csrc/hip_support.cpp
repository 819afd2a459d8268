// Everything in the library that talks to the HIP runtime outside the kernels: the driver-operation
// tables of the memory manager (virtual-memory calls, or plain hipMalloc for the statically backed
// baseline), the pinned staging ring, the kernel timers and the virtual-memory micro-benchmark.
#include <chrono>
#include <cstdio>

#include "vattn_internal.h"

namespace vattn {

bool hip_ok(hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    (void)hipGetLastError();  // clear the sticky error so later calls are not blamed for it
    return false;
}

namespace {

double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

hipMemAllocationProp device_prop(int device) {
    hipMemAllocationProp prop{};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    return prop;
}

static_assert(sizeof(hipMemGenericAllocationHandle_t) <= sizeof(uint64_t), "handles are stored as 64-bit values");
hipMemGenericAllocationHandle_t as_handle(uint64_t h) { return reinterpret_cast<hipMemGenericAllocationHandle_t>(h); }

bool op_bind(int device) { return hip_ok(hipSetDevice(device), "hipSetDevice"); }
bool op_device_sync() { return hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize"); }

// ---- Sec. 5.2.1 of the paper: the virtual-memory calls (Table 3), in their HIP spelling ------------
bool vmm_granularity(int device, size_t* bytes) {
    int vmm = 0;
    if (!hip_ok(hipDeviceGetAttribute(&vmm, hipDeviceAttributeVirtualMemoryManagementSupported, device), "hipDeviceGetAttribute")) return false;
    if (!vmm) { set_error("init: device does not support virtual memory management"); return false; }
    const hipMemAllocationProp prop = device_prop(device);
    return hip_ok(hipMemGetAllocationGranularity(bytes, &prop, hipMemAllocationGranularityMinimum), "hipMemGetAllocationGranularity");
}
bool vmm_reserve(void** va, size_t bytes, size_t align) { return hip_ok(hipMemAddressReserve(va, bytes, align, nullptr, 0), "hipMemAddressReserve"); }
bool vmm_va_free(void* va, size_t bytes) { return hip_ok(hipMemAddressFree(va, bytes), "hipMemAddressFree"); }
bool vmm_create(uint64_t* handle, size_t bytes, int device) {
    const hipMemAllocationProp prop = device_prop(device);
    hipMemGenericAllocationHandle_t h;
    if (!hip_ok(hipMemCreate(&h, bytes, &prop, 0), "hipMemCreate (physical pool)")) return false;
    *handle = reinterpret_cast<uint64_t>(h);
    return true;
}
bool vmm_release(uint64_t handle) { return hip_ok(hipMemRelease(as_handle(handle)), "hipMemRelease"); }
bool vmm_map(void* va, size_t bytes, uint64_t handle) { return hip_ok(hipMemMap(va, bytes, 0, as_handle(handle), 0), "hipMemMap"); }
bool vmm_set_access(void* va, size_t bytes, int device) {
    hipMemAccessDesc d{};
    d.location.type = hipMemLocationTypeDevice;
    d.location.id = device;
    d.flags = hipMemAccessFlagsProtReadWrite;
    return hip_ok(hipMemSetAccess(va, bytes, &d, 1), "hipMemSetAccess");
}
bool vmm_unmap(void* va, size_t bytes) { return hip_ok(hipMemUnmap(va, bytes), "hipMemUnmap"); }

// How many page-group handles one pool may hold: pools of 65 536 handles and more were seen to crash the process
// inside the runtime on MI355X (with 4 KiB and with 64 KiB handles, during creation or mapping), while 27 648
// handles worked.  Measured since: hipMemCreate adds no memory mapping and no file descriptor to the process,
// and the machine measured allows 1 048 576 mappings - so neither the cap on mappings (65 530 by default, which
// is what the threshold looked like) nor the descriptor limit explains it.  The cause is still unknown, the
// case was not run again, and the library keeps refusing more than 32 768.  Larger caches need
// larger page-groups: 32 768 x 2 MiB = 64 GiB, x 16 MiB = 512 GiB.
int64_t vmm_mapping_limit() { return 32768; }
// Measured on MI355X / ROCm 7.2: in a process whose first user of the runtime is this library, hipMemMap adds
// 1.00-1.07 memory mappings of the process per page-group (none in a process where PyTorch initialised the
// runtime first), hipMemCreate and hipMemSetAccess none, and hipMemUnmap / hipMemRelease remove none - they only
// go away with hipMemAddressFree.  So what can count against vm.max_map_count is every (buffer, page-group)
// address that was EVER mapped; the budget assumes the dearer case and leaves room for the rest of the process
// and for the 7 % on top.
int64_t vmm_mapping_budget() {
    long v = 65530;
    if (FILE* f = std::fopen("/proc/sys/vm/max_map_count", "r")) {
        long x = 0;
        if (std::fscanf(f, "%ld", &x) == 1 && x > 0) v = x;
        std::fclose(f);
    }
    const long headroom = 16384;
    const long usable = v > 2 * headroom ? v - headroom : v / 2;
    return static_cast<int64_t>(usable / 1.1);
}
int64_t no_mapping_limit() { return 0; }

// ---- statically backed baseline: the whole buffer is allocated up front, mapping is bookkeeping ----
bool static_granularity(int, size_t* bytes) { *bytes = 4096; return true; }
bool static_reserve(void** va, size_t bytes, size_t) { return hip_ok(hipMalloc(va, bytes), "hipMalloc (statically backed KV buffer)"); }
bool static_va_free(void* va, size_t) { return hip_ok(hipFree(va), "hipFree"); }
bool static_create(uint64_t* handle, size_t, int) { static uint64_t next = 1; *handle = next++; return true; }
bool static_release(uint64_t) { return true; }
bool static_map(void*, size_t, uint64_t) { return true; }
bool static_set_access(void*, size_t, int) { return true; }
bool static_unmap(void*, size_t) { return true; }

}  // namespace

const VmmOps& hip_vmm_ops() {
    static const VmmOps ops{op_bind, vmm_granularity, vmm_reserve, vmm_va_free, vmm_create, vmm_release,
                            vmm_map, vmm_set_access, vmm_unmap, op_device_sync, vmm_mapping_limit, vmm_mapping_budget};
    return ops;
}

const VmmOps& hip_static_ops() {
    static const VmmOps ops{op_bind, static_granularity, static_reserve, static_va_free, static_create, static_release,
                            static_map, static_set_access, static_unmap, op_device_sync, no_mapping_limit, no_mapping_limit};
    return ops;
}

// ---------------------------------------------------------------------------------------------
// Per-call latency of the virtual-memory API (the analogue of Table 3 of the paper), measured on
// `count` page-groups of `bytes` each: out_us[0..8] = average microseconds of
//   0 hipMemAddressReserve (one range for all)   1 hipMemCreate        2 hipMemMap
//   3 hipMemSetAccess, one call per page-group   4 hipMemSetAccess, ONE call over all (total time)
//   5 hipMemUnmap                                6 hipMemRelease       7 hipMemAddressFree
//   8 a fill kernel touching every mapped byte once (total, microseconds) - proves the mapping is usable.
// out_us[9..11] are not times: memory mappings of the process (lines of /proc/self/maps) added per hipMemCreate,
// added per hipMemMap, and given back per hipMemUnmap.
// ---------------------------------------------------------------------------------------------
// Memory mappings of this process (lines of /proc/self/maps); -1 if unreadable.
static long process_mappings() {
    FILE* f = std::fopen("/proc/self/maps", "r");
    if (!f) return -1;
    long n = 0;
    for (int c; (c = std::fgetc(f)) != EOF;) n += c == '\n';
    std::fclose(f);
    return n;
}

__global__ void touch_kernel(uint32_t* p, size_t n) {
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n; i += static_cast<size_t>(gridDim.x) * blockDim.x) p[i] = static_cast<uint32_t>(i);
}

bool vmm_microbench(int device, int64_t bytes, int count, double* out_us) {
    if (bytes <= 0 || count <= 0 || !out_us) { set_error("vmm_microbench: invalid argument"); return false; }
    if (!op_bind(device)) return false;
    size_t gran = 0;
    if (!vmm_granularity(device, &gran)) return false;
    if (bytes % static_cast<int64_t>(gran) != 0) { set_error("vmm_microbench: size must be a multiple of the granularity (" + std::to_string(gran) + ")"); return false; }
    const size_t G = static_cast<size_t>(bytes), total = G * static_cast<size_t>(count);
    for (int i = 0; i < 12; ++i) out_us[i] = 0;
    void* va = nullptr;
    double t = now_us();
    if (!vmm_reserve(&va, total, G)) return false;
    out_us[0] = now_us() - t;
    char* base = static_cast<char*>(va);
    std::vector<uint64_t> h(static_cast<size_t>(count), 0);
    int created = 0, mapped = 0;
    bool ok = true;
    const long maps0 = process_mappings();
    t = now_us();
    for (; created < count && ok; ++created) ok = vmm_create(&h[created], G, device);
    if (!ok) --created;
    out_us[1] = (now_us() - t) / count;
    const long maps1 = process_mappings();
    out_us[9] = static_cast<double>(maps1 - maps0) / count;
    if (ok) {
        t = now_us();
        for (; mapped < count && ok; ++mapped) ok = vmm_map(base + static_cast<size_t>(mapped) * G, G, h[mapped]);
        if (!ok) --mapped;
        out_us[2] = (now_us() - t) / count;
        out_us[10] = static_cast<double>(process_mappings() - maps1) / count;
    }
    if (ok) {
        t = now_us();
        for (int i = 0; i < count && ok; ++i) ok = vmm_set_access(base + static_cast<size_t>(i) * G, G, device);
        out_us[3] = (now_us() - t) / count;
    }
    if (ok) {   // the same range again, freshly mapped, made accessible by ONE call
        for (int i = 0; i < count; ++i) (void)vmm_unmap(base + static_cast<size_t>(i) * G, G);
        mapped = 0;
        for (; mapped < count && ok; ++mapped) ok = vmm_map(base + static_cast<size_t>(mapped) * G, G, h[mapped]);
        if (!ok) --mapped;
        if (ok) {
            t = now_us();
            ok = vmm_set_access(base, total, device);
            out_us[4] = now_us() - t;
        }
    }
    if (ok) {   // every access above succeeded, so the whole range is readable and writable
        ok = op_device_sync();
        t = now_us();
        hipLaunchKernelGGL(touch_kernel, dim3(1024), dim3(256), 0, nullptr, reinterpret_cast<uint32_t*>(base), total / 4);
        ok = ok && hip_ok(hipGetLastError(), "touch kernel launch") && op_device_sync();
        out_us[8] = now_us() - t;
    }
    const std::string first_error = ok ? std::string() : last_error_string();
    const long maps2 = process_mappings();
    t = now_us();
    for (int i = 0; i < mapped; ++i) (void)vmm_unmap(base + static_cast<size_t>(i) * G, G);
    out_us[5] = mapped ? (now_us() - t) / mapped : 0;
    out_us[11] = mapped ? static_cast<double>(maps2 - process_mappings()) / mapped : 0;
    t = now_us();
    for (int i = 0; i < created; ++i) (void)vmm_release(h[i]);
    out_us[6] = created ? (now_us() - t) / created : 0;
    t = now_us();
    (void)vmm_va_free(va, total);
    out_us[7] = now_us() - t;
    if (!ok) { set_error(first_error); return false; }
    return true;
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
    // Until release() records the slot's event the slot counts as busy up to this point of the stream.
    if (!hip_ok(hipEventRecord(ev_[cur_], stream), "hipEventRecord")) return false;
    pending_[cur_] = true;
    return true;
}

bool MetaRing::release(hipStream_t stream) {
    if (cur_ < 0 || !pending_[cur_]) return true;
    return hip_ok(hipEventRecord(ev_[cur_], stream), "hipEventRecord");
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
