// Host-only driver of the KV memory manager: the driver-operation table is filled with bookkeeping
// fakes (no GPU runtime), commands come from stdin, the manager's state goes to stdout.  Built with a
// plain C++ compiler (optionally with a thread sanitizer) by tests/test_host_manager.py.
//
// Commands:  init N B L H D G pool flags lookahead eager threshold | a | f <reqid> | s <len>*B | q | quit
//            fail <reserve|create|map|access> <k>   the k-th call of that operation from now on fails, once
//            budget <n>   the next init gets a cap of n distinct (buffer, page-group) address slots | err
#include <cstdio>
#include <iostream>
#include <map>
#include <mutex>
#include <set>
#include <sstream>
#include <string>

#include "../../paper_2405_04437_amd/csrc/kv_memory.h"

namespace {

// The fakes keep their own record of what is mapped where, and fail on anything the real driver would
// reject: mapping over a mapped range, mapping a handle twice, unmapping what is not mapped.
std::mutex g_mu;
std::map<uintptr_t, uint64_t> g_mapped;   // va -> handle
std::set<uint64_t> g_in_use, g_alive;
std::set<uintptr_t> g_access;
uintptr_t g_next_va = uintptr_t{1} << 40;
uint64_t g_next_handle = 1;
long g_violations = 0;
size_t g_G = 0;

bool bad(const char* what) { ++g_violations; vattn::set_error(what); return false; }

// Injected driver failures: countdown per operation (0 = none armed); the call that takes it to zero fails.
enum { kReserve, kCreate, kMap, kAccess, kOps };
long g_fail_in[kOps] = {};
bool injected(int op, const char* what) {
    if (g_fail_in[op] > 0 && --g_fail_in[op] == 0) { vattn::set_error(std::string("injected failure: ") + what); return true; }
    return false;
}

bool f_bind(int) { return true; }
bool f_gran(int, size_t* b) { *b = 4096; return true; }
bool f_reserve(void** va, size_t bytes, size_t align) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (injected(kReserve, "reserve")) return false;
    g_next_va = (g_next_va + align - 1) / align * align;
    *va = reinterpret_cast<void*>(g_next_va);
    g_next_va += bytes;
    return true;
}
bool f_va_free(void*, size_t) { return true; }
bool f_create(uint64_t* h, size_t bytes, int) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (injected(kCreate, "create")) return false;
    g_G = bytes;
    *h = g_next_handle++;
    g_alive.insert(*h);
    return true;
}
bool f_release(uint64_t h) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_in_use.count(h)) return bad("release of a mapped handle");
    return g_alive.erase(h) == 1 ? true : bad("release of an unknown handle");
}
bool f_map(void* va, size_t bytes, uint64_t h) {
    std::lock_guard<std::mutex> lk(g_mu);
    const uintptr_t a = reinterpret_cast<uintptr_t>(va);
    if (injected(kMap, "map")) return false;
    if (bytes != g_G || a % g_G) return bad("map: wrong size or alignment");
    if (!g_alive.count(h)) return bad("map: unknown handle");
    if (g_in_use.count(h)) return bad("map: handle already mapped");
    if (g_mapped.count(a)) return bad("map: range already mapped");
    g_mapped[a] = h;
    g_in_use.insert(h);
    return true;
}
bool f_access(void* va, size_t bytes, int) {
    std::lock_guard<std::mutex> lk(g_mu);
    const uintptr_t a = reinterpret_cast<uintptr_t>(va);
    if (injected(kAccess, "access")) return false;
    for (uintptr_t x = a; x < a + bytes; x += g_G) {
        if (!g_mapped.count(x)) return bad("set_access over an unmapped range");
        g_access.insert(x);
    }
    return true;
}
bool f_unmap(void* va, size_t bytes) {
    std::lock_guard<std::mutex> lk(g_mu);
    const uintptr_t a = reinterpret_cast<uintptr_t>(va);
    auto it = g_mapped.find(a);
    if (bytes != g_G || it == g_mapped.end()) return bad("unmap of an unmapped range");
    g_in_use.erase(it->second);
    g_mapped.erase(it);
    g_access.erase(a);
    return true;
}
bool f_sync() { return true; }
long g_budget = 0;   // distinct address slots the next context may map over its life (0 = unlimited)
int64_t f_budget() { return g_budget; }

}  // namespace

int main() {
    const vattn::VmmOps ops{f_bind, f_gran, f_reserve, f_va_free, f_create, f_release, f_map, f_access, f_unmap, f_sync, nullptr, f_budget};
    vattn::KvMemory* mem = nullptr;
    vattn_config cfg{};
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
        std::string cmd;
        in >> cmd;
        if (cmd == "init") {
            long long L, G, pool, thr;
            unsigned flags;
            in >> cfg.num_layers >> cfg.max_batch >> L >> cfg.num_kv_heads >> cfg.head_dim >> G >> pool >> flags >> cfg.lookahead_tokens >> cfg.eager_page_groups >> thr;
            cfg.max_ctx = L; cfg.num_q_heads = cfg.num_kv_heads; cfg.elem_bytes = 2; cfg.page_group_bytes = G;
            cfg.phys_budget_bytes = pool * G; cfg.flags = flags; cfg.reclaim_threshold_page_groups = thr;
            delete mem;
            mem = new vattn::KvMemory();
            const bool ok = mem->init(cfg, ops);
            std::printf("%d\n", ok ? 0 : -1);
            if (!ok) { delete mem; mem = nullptr; }
        } else if (cmd == "a") {
            std::printf("%d\n", mem->alloc_reqid());
        } else if (cmd == "f") {
            int r; in >> r;
            std::printf("%d\n", mem->free_reqid(r));
        } else if (cmd == "s") {
            std::vector<int64_t> lens;
            long long x;
            while (in >> x) lens.push_back(x);
            std::printf("%d\n", mem->step(lens.data(), static_cast<int>(lens.size())));
        } else if (cmd == "q") {
            const vattn::KvMemory::Counters c = mem->counters();
            std::printf("free %lld maps %lld unmaps %lld sync %lld bg %lld S %lld viol %ld live %zu |",
                        (long long)mem->pool_free(), (long long)c.map_calls, (long long)c.unmap_calls, (long long)c.sync_map_calls,
                        (long long)c.background_map_calls, (long long)mem->S(), g_violations, g_mapped.size());
            for (int r = 0; r < cfg.max_batch; ++r) std::printf(" %d:%lld:%lld", mem->is_active(r) ? 1 : 0, (long long)mem->mapped(r), (long long)mem->mapped_committed(r));
            std::printf("\n");
        } else if (cmd == "fail") {
            std::string op; long k = 0;
            in >> op >> k;
            const int which = op == "reserve" ? kReserve : op == "create" ? kCreate : op == "map" ? kMap : op == "access" ? kAccess : -1;
            if (which >= 0) g_fail_in[which] = k;
            std::printf("%d\n", which >= 0 ? 0 : -1);
        } else if (cmd == "budget") {
            in >> g_budget;
            std::printf("0\n");
        } else if (cmd == "err") {
            std::printf("%s\n", vattn::last_error_string().c_str());
        } else if (cmd == "quit") {
            break;
        }
        std::fflush(stdout);
    }
    delete mem;
    std::printf("end viol %ld live %zu alive %zu\n", g_violations, g_mapped.size(), g_alive.size());
    return g_violations ? 1 : 0;
}
