// KV-cache memory manager: bookkeeping of virtual buffers, physical page-groups and reqIds.
//
// This header and kv_memory.cpp contain no GPU runtime call: the seven driver operations the manager
// needs are reached through a table of function pointers (VmmOps).  The library fills the table with
// the HIP virtual-memory calls; a host-only build can fill it with counters, which is how the manager
// and its background thread are exercised under a thread sanitizer on a machine without a GPU.
#pragma once

#include <condition_variable>
#include <cstddef>
#include <cstdint>
#include <functional>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/vattn.h"

namespace vattn {

void set_error(const std::string& msg);
const std::string& last_error_string();

// Driver operations.  Each returns false on failure after recording a message with set_error().
struct VmmOps {
    bool (*bind_thread)(int device);                               // make `device` current on this thread
    bool (*granularity)(int device, size_t* bytes);                // minimum size/alignment of a physical handle
    bool (*reserve)(void** va, size_t bytes, size_t align);        // virtual address range, nothing behind it
    bool (*va_free)(void* va, size_t bytes);
    bool (*create)(uint64_t* handle, size_t bytes, int device);    // one physical page-group
    bool (*release)(uint64_t handle);
    bool (*map)(void* va, size_t bytes, uint64_t handle);          // handle -> va (offset 0, whole handle)
    bool (*set_access)(void* va, size_t bytes, int device);        // read/write for the device
    bool (*unmap)(void* va, size_t bytes);
    bool (*device_sync)();                                         // wait for all work queued on the device
    int64_t (*mapping_limit)();                                    // most page-group handles one pool may hold (0 = no limit)
    // How many DISTINCT (buffer, page-group) address slots a context may map over its whole life (0 = no limit):
    // on Linux every slot that was ever mapped stays a separate memory mapping of the process until the
    // reservation is freed - unmapping does not give it back - and the system caps their number.
    int64_t (*mapping_budget)();
};

// One helper thread that runs one task at a time.  submit() and wait() are called from the thread
// that owns the manager; wait() returning gives that thread a happens-before edge from the task.
class Worker {
public:
    ~Worker();
    void start(std::function<void()> on_start);
    void submit(std::function<void()> task);
    void wait();
    bool running() const { return thread_.joinable(); }

private:
    void loop(std::function<void()> on_start);
    std::thread thread_;
    std::mutex mu_;
    std::condition_variable cv_;
    std::function<void()> task_;
    bool busy_ = false, stop_ = false;
};

// Follows Sec. 5 of the paper (virtual tensors, reqId indexing, init/alloc_reqid/free_reqid/step),
// Sec. 6.1 (background thread: look-ahead mapping, deferred reclamation, eager allocation) and the
// tensor-slicing layout of its discussion section.
class KvMemory {
public:
    ~KvMemory();
    bool init(const vattn_config& cfg, const VmmOps& ops);
    int alloc_reqid();
    int free_reqid(int reqid);
    int step(const int64_t* seq_lens, int count);
    // Joins the background pass, if one is running, and publishes its result.  Every call that reads or
    // changes the bookkeeping goes through here first; the kernel launchers do not (see mapped_committed).
    void sync();

    // Layer `layer`, K (which = 0) or V (1): address of token 0 of reqId 0.  Consecutive reqIds are S bytes
    // apart, consecutive tokens token_stride() bytes (H*D*P, or N*H*D*P when all layers share a buffer).
    char* buffer_base(int layer, int which) const {
        return sliced_ ? base_[which] + static_cast<int64_t>(layer) * T_ : base_[static_cast<size_t>(layer) * 2 + which];
    }
    char* sub_tensor(int layer, int which, int reqid) const { return buffer_base(layer, which) + static_cast<int64_t>(reqid) * S_; }
    bool valid_reqid(int r) const { return r >= 0 && r < B_; }
    bool is_active(int r) const { return active_[r] != 0; }          // changed only by the owning thread
    // Page-groups known to be mapped under reqId r as of the last sync(): a lower bound of the truth
    // while a background pass runs, which is what launch-time validation needs.
    int64_t mapped_committed(int r) const { return committed_[r]; }
    int64_t mapped(int r) { sync(); return mapped_[r]; }
    int64_t G() const { return G_; }
    int64_t S() const { return S_; }
    int64_t T() const { return T_; }
    int64_t token_stride() const { return Tbuf_; }
    int num_buffers() const { return nbuf_; }
    int64_t pool_total() const { return pool_total_; }
    int64_t pool_free() { sync(); return static_cast<int64_t>(free_handles_.size()); }

    struct Counters {
        int64_t map_calls = 0, unmap_calls = 0;            // (buffer, page-group) operations, all threads
        int64_t sync_map_calls = 0, background_map_calls = 0;
        double map_us = 0, unmap_us = 0;                   // wall time inside the driver calls
        double step_us = 0;                                // wall time of step() calls on the caller's thread
        double background_us = 0;                          // wall time of background passes
        double wait_us = 0;                                // time the caller spent waiting for a background pass
    };
    Counters counters() { sync(); return c_; }

private:
    bool map_rows(int r, int64_t from, int64_t to, bool background);  // page-group rows [from,to) of reqId r, all buffers
    void unmap_rows(int r, int64_t keep);                             // unmap rows [keep, mapped) and return handles
    int64_t need(int64_t tokens) const { return (tokens * Tbuf_ + G_ - 1) / G_; }   // (s + t - 1) / t
    int next_candidate() const;
    void background_pass(const std::vector<int64_t>& lens);
    int64_t free_now() const { return static_cast<int64_t>(free_handles_.size()); }

    VmmOps ops_{};
    int N_ = 0, B_ = 0, device_ = 0, nbuf_ = 0;
    uint32_t policy_ = 0;
    bool sliced_ = false, background_ = false;
    int64_t lookahead_ = 0, eager_ = 0, reclaim_threshold_ = 0;
    int64_t L_ = 0, G_ = 0, S_ = 0, T_ = 0, Tbuf_ = 0, pool_total_ = 0;
    std::vector<char*> base_;                          // reservations of B*S bytes
    std::vector<uint64_t> free_handles_;               // created, unmapped
    std::vector<std::vector<uint64_t>> held_;          // per reqId: rows x buffers handles
    std::vector<uint8_t> active_;
    std::vector<int64_t> mapped_;                      // owned by whichever thread currently runs (caller or pass)
    std::vector<int64_t> high_water_;                  // per reqId: most rows ever mapped (each row touched nbuf_ address slots)
    int64_t touched_ = 0, budget_ = 0;                 // address slots mapped at least once, and their cap (0 = none)
    std::vector<int64_t> committed_;                   // copy of mapped_ taken at sync(), read by launch validation
    Counters c_;
    Worker worker_;
    bool pass_pending_ = false;
};

}  // namespace vattn
