// KV-cache memory manager (bookkeeping; see kv_memory.h).
//
// Design (Sec. 5 of the paper, re-expressed for HIP): virtual address space is reserved once for the
// largest batch and context, physical page-groups are created up front but mapped only when step()
// sees that a request's context has outgrown what is backed.  One physical handle per page-group: HIP
// rejects mapping a handle at a non-zero offset, so a page-group is the unit of both creation and
// mapping.  With the background option (Sec. 6.1) a helper thread maps the next iteration's growth,
// prepares the next reqId and reclaims deferred pages while the caller runs the current iteration.
#include "kv_memory.h"

#include <algorithm>
#include <chrono>

namespace vattn {

namespace {
thread_local std::string g_error;
double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
}  // namespace

void set_error(const std::string& msg) { g_error = msg; }
const std::string& last_error_string() { return g_error; }

// ---------------------------------------------------------------------------------------------

Worker::~Worker() {
    if (!thread_.joinable()) return;
    {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return !busy_; });
        stop_ = true;
    }
    cv_.notify_all();
    thread_.join();
}

void Worker::start(std::function<void()> on_start) {
    thread_ = std::thread([this, on_start] { loop(on_start); });
}

void Worker::loop(std::function<void()> on_start) {
    if (on_start) on_start();
    std::unique_lock<std::mutex> lk(mu_);
    for (;;) {
        cv_.wait(lk, [&] { return stop_ || busy_; });
        if (stop_) return;
        std::function<void()> t = std::move(task_);
        task_ = nullptr;
        lk.unlock();
        t();
        lk.lock();
        busy_ = false;
        cv_.notify_all();
    }
}

void Worker::submit(std::function<void()> task) {
    {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return !busy_; });
        task_ = std::move(task);
        busy_ = true;
    }
    cv_.notify_all();
}

void Worker::wait() {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return !busy_; });
}

// ---------------------------------------------------------------------------------------------

bool KvMemory::init(const vattn_config& c, const VmmOps& ops) {
    ops_ = ops;
    if (c.num_layers <= 0 || c.max_batch <= 0 || c.max_ctx <= 0 || c.num_kv_heads <= 0 ||
        c.num_q_heads <= 0 || c.num_q_heads % c.num_kv_heads != 0) {
        set_error("init: N, B, L, H must be positive and Hq a multiple of H");
        return false;
    }
    if (c.head_dim != 64 && c.head_dim != 128) { set_error("init: head_dim must be 64 or 128"); return false; }
    if (c.elem_bytes != 2) { set_error("init: only 2-byte (bf16) elements are supported"); return false; }
    const uint32_t known = VATTN_POLICY_MASK | VATTN_FLAG_BACKGROUND | VATTN_FLAG_STATIC_BACKING | VATTN_FLAG_TENSOR_SLICING;
    policy_ = c.flags & VATTN_POLICY_MASK;
    if ((c.flags & ~known) != 0 || (policy_ != VATTN_POLICY_SYNC_UNMAP && policy_ != VATTN_POLICY_DEFERRED)) {
        set_error("init: unknown policy or flag bits");
        return false;
    }
    if (c.lookahead_tokens < 0 || c.eager_page_groups < 0 || c.reclaim_threshold_page_groups < 0) {
        set_error("init: negative look-ahead, eager or threshold value");
        return false;
    }
    device_ = c.device;
    if (!ops_.bind_thread(device_)) return false;
    size_t gran = 0;
    if (!ops_.granularity(device_, &gran)) return false;
    if (gran == 0) { set_error("init: zero allocation granularity"); return false; }
    int64_t G = c.page_group_bytes == 0 ? (int64_t{2} << 20) : c.page_group_bytes;
    if (c.page_group_bytes == 0) G = (G + static_cast<int64_t>(gran) - 1) / static_cast<int64_t>(gran) * static_cast<int64_t>(gran);
    if (G <= 0 || G % static_cast<int64_t>(gran) != 0) {
        set_error("init: page_group_bytes must be a positive multiple of the allocation granularity (" + std::to_string(gran) + ")");
        return false;
    }
    N_ = c.num_layers; B_ = c.max_batch; L_ = c.max_ctx; G_ = G;
    sliced_ = (c.flags & VATTN_FLAG_TENSOR_SLICING) != 0;
    background_ = (c.flags & VATTN_FLAG_BACKGROUND) != 0;
    lookahead_ = c.lookahead_tokens; eager_ = c.eager_page_groups; reclaim_threshold_ = c.reclaim_threshold_page_groups;
    nbuf_ = sliced_ ? 2 : 2 * N_;
    T_ = static_cast<int64_t>(c.num_kv_heads) * c.head_dim * c.elem_bytes;
    Tbuf_ = sliced_ ? T_ * N_ : T_;
    if (L_ > (int64_t{1} << 40) / Tbuf_) { set_error("init: L*H*D*P does not fit the address arithmetic"); return false; }
    if (L_ > int64_t{0x7FFFFF00}) { set_error("init: L must stay below 2^31 tokens (the kernels count tokens in 32 bits)"); return false; }
    S_ = (L_ * Tbuf_ + G_ - 1) / G_ * G_;
    pool_total_ = c.phys_budget_bytes / G_;
    if (pool_total_ < 0) { set_error("init: negative physical budget"); return false; }
    const int64_t limit = ops_.mapping_limit ? ops_.mapping_limit() : 0;
    if (limit > 0 && pool_total_ > limit) {
        set_error("init: the pool has " + std::to_string(pool_total_) + " page-groups, but the limit is " +
                  std::to_string(limit) + " (very large handle counts are not safe on this platform); use larger page-groups");
        return false;
    }

    // The per-reqId tables exist before the first driver call: if a reservation or a handle creation below
    // fails, the destructor finds a consistent (empty) state and releases what was made so far.
    held_.assign(static_cast<size_t>(B_), {});
    high_water_.assign(static_cast<size_t>(B_), 0);
    touched_ = 0;
    budget_ = ops_.mapping_budget ? ops_.mapping_budget() : 0;
    active_.assign(static_cast<size_t>(B_), 0);
    mapped_.assign(static_cast<size_t>(B_), 0);
    committed_.assign(static_cast<size_t>(B_), 0);
    const size_t buf_bytes = static_cast<size_t>(B_) * static_cast<size_t>(S_);
    base_.assign(static_cast<size_t>(nbuf_), nullptr);
    for (size_t b = 0; b < base_.size(); ++b) {
        void* p = nullptr;
        if (!ops_.reserve(&p, buf_bytes, static_cast<size_t>(G_))) return false;
        base_[b] = static_cast<char*>(p);
    }
    free_handles_.reserve(static_cast<size_t>(pool_total_));
    for (int64_t i = 0; i < pool_total_; ++i) {
        uint64_t h = 0;
        if (!ops_.create(&h, static_cast<size_t>(G_), device_)) return false;
        free_handles_.push_back(h);
    }
    if (background_) {
        const VmmOps o = ops_;
        const int dev = device_;
        worker_.start([o, dev] { (void)o.bind_thread(dev); });
    }
    return true;
}

KvMemory::~KvMemory() {
    if (base_.empty()) return;
    sync();
    (void)ops_.bind_thread(device_);
    (void)ops_.device_sync();
    for (int r = 0; r < static_cast<int>(mapped_.size()); ++r) unmap_rows(r, 0);
    for (auto h : free_handles_) (void)ops_.release(h);
    const size_t buf_bytes = static_cast<size_t>(B_) * static_cast<size_t>(S_);
    for (char* p : base_) if (p) (void)ops_.va_free(p, buf_bytes);
}

void KvMemory::sync() {
    if (!pass_pending_) return;
    const double t0 = now_us();
    worker_.wait();
    c_.wait_us += now_us() - t0;
    pass_pending_ = false;
    committed_ = mapped_;
}

int KvMemory::next_candidate() const {
    int best = -1;
    for (int r = 0; r < B_; ++r) {
        if (active_[r]) continue;
        if (best < 0) { best = r; if (policy_ == VATTN_POLICY_SYNC_UNMAP) break; continue; }
        if (mapped_[r] > mapped_[best]) best = r;  // most pages still mapped; ties keep the lowest id
    }
    return best;
}

int KvMemory::alloc_reqid() {
    sync();
    const int best = next_candidate();
    if (best < 0) { set_error("alloc_reqid: all reqIds are in use"); return -1; }
    active_[best] = 1;
    return best;
}

int KvMemory::free_reqid(int r) {
    sync();
    if (!valid_reqid(r) || !active_[r]) { set_error("free_reqid: reqId out of range or not active"); return -1; }
    active_[r] = 0;
    if (policy_ == VATTN_POLICY_SYNC_UNMAP) { unmap_rows(r, 0); committed_[r] = 0; }
    return 0;
}

bool KvMemory::map_rows(int r, int64_t from, int64_t to, bool background) {
    const size_t nb = base_.size();
    auto& held = held_[r];
    const double t0 = now_us();
    if (budget_ > 0 && to > high_water_[r] && touched_ + (to - std::max(high_water_[r], from)) * static_cast<int64_t>(nb) > budget_) {
        set_error("mapping " + std::to_string(to - from) + " more page-group rows of reqId " + std::to_string(r) + " would exceed the " +
                  std::to_string(budget_) + " distinct address slots this process may map (the system's cap on memory mappings; "
                  "a slot stays a mapping after it is unmapped): use larger page-groups or a smaller B*L");
        return false;
    }
    for (int64_t k = from; k < to; ++k) {
        if (k + 1 > high_water_[r]) { high_water_[r] = k + 1; touched_ += static_cast<int64_t>(nb); }
        for (size_t b = 0; b < nb; ++b) {
            const uint64_t h = free_handles_.back();
            char* va = base_[b] + static_cast<int64_t>(r) * S_ + k * G_;
            if (!ops_.map(va, static_cast<size_t>(G_), h)) {
                // undo the partial row and everything mapped by this call
                for (size_t u = 0; u < b; ++u) {
                    (void)ops_.unmap(base_[u] + static_cast<int64_t>(r) * S_ + k * G_, static_cast<size_t>(G_));
                    free_handles_.push_back(held.back()); held.pop_back();
                }
                mapped_[r] = k; unmap_rows(r, from);
                return false;
            }
            free_handles_.pop_back();
            held.push_back(h);
            ++c_.map_calls;
            ++(background ? c_.background_map_calls : c_.sync_map_calls);
        }
        mapped_[r] = k + 1;
    }
    // One access call per buffer covers the whole newly mapped, contiguous range.
    for (size_t b = 0; b < nb; ++b) {
        char* va = base_[b] + static_cast<int64_t>(r) * S_ + from * G_;
        if (!ops_.set_access(va, static_cast<size_t>((to - from) * G_), device_)) {
            unmap_rows(r, from);
            return false;
        }
    }
    c_.map_us += now_us() - t0;
    return true;
}

void KvMemory::unmap_rows(int r, int64_t keep) {
    const size_t nb = base_.size();
    auto& held = held_[r];
    const double t0 = now_us();
    for (int64_t k = mapped_[r] - 1; k >= keep; --k) {
        for (size_t b = nb; b-- > 0;) {
            (void)ops_.unmap(base_[b] + static_cast<int64_t>(r) * S_ + k * G_, static_cast<size_t>(G_));
            free_handles_.push_back(held.back());
            held.pop_back();
            ++c_.unmap_calls;
        }
    }
    if (mapped_[r] > keep) mapped_[r] = keep;
    c_.unmap_us += now_us() - t0;
}

int KvMemory::step(const int64_t* seq_lens, int count) {
    const double t_begin = now_us();
    sync();
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
        const int64_t nd = need(n);
        want[r] = nd > mapped_[r] ? nd : mapped_[r];
        demand_rows += want[r] - mapped_[r];
    }
    const int64_t per_row = nbuf_;
    const int64_t demand = demand_rows * per_row;
    if (budget_ > 0) {   // rows that were never mapped before take new address slots
        int64_t fresh = 0;
        for (int r = 0; r < B_; ++r)
            if (active_[r] && want[r] > high_water_[r]) fresh += want[r] - std::max(high_water_[r], mapped_[r]);
        if (touched_ + fresh * per_row > budget_) {
            set_error("step: " + std::to_string(fresh * per_row) + " page-groups at addresses never mapped before would exceed the " +
                      std::to_string(budget_) + " distinct address slots this process may map (the system's cap on memory mappings; "
                      "a slot stays a mapping after it is unmapped): use larger page-groups or a smaller B*L");
            return -1;
        }
    }
    if (demand > free_now() + reclaimable_rows * per_row) {
        set_error("step: physical pool exhausted (demand " + std::to_string(demand) + " page-groups, free " + std::to_string(free_now()) + ")");
        return -1;
    }
    // What this call changes, so that a failing driver call can be rolled back: the mapped count of every reqId
    // at entry (active ones grow, inactive ones may be reclaimed from).
    const std::vector<int64_t> before = mapped_;
    if (demand > free_now()) {  // deferred policy: take pages back from inactive ids, lowest id first
        // A request that was freed a moment ago may still be read by a kernel that is enqueued or running:
        // nothing is unmapped before the device has drained (rare path - only when the pool is short).
        (void)ops_.device_sync();
        for (int r = 0; r < B_ && free_now() < demand; ++r) {
            if (active_[r]) continue;
            while (mapped_[r] > 0 && free_now() < demand) unmap_rows(r, mapped_[r] - 1);
        }
    }
    int rc = 0;
    for (int r = 0; r < B_; ++r) {
        if (!active_[r] || want[r] <= mapped_[r]) continue;
        if (!map_rows(r, mapped_[r], want[r], false)) { rc = -1; break; }
    }
    if (rc != 0) {
        // A driver call failed (map_rows has already undone its own request).  All-or-nothing: the requests
        // that grew earlier in this call shrink back, then the page-groups reclaimed from inactive ids are
        // mapped again - if the driver refuses that too they stay in the pool, which an inactive id may not
        // rely on anyway.  The error text of the first failure is kept.
        const std::string first = last_error_string();
        for (int r = 0; r < B_; ++r)
            if (active_[r] && mapped_[r] > before[r]) unmap_rows(r, before[r]);
        for (int r = 0; r < B_; ++r)
            if (!active_[r] && mapped_[r] < before[r] && (before[r] - mapped_[r]) * per_row <= free_now())
                (void)map_rows(r, mapped_[r], before[r], false);
        set_error(first);
    }
    committed_ = mapped_;
    if (rc == 0 && background_) {
        std::vector<int64_t> lens(seq_lens, seq_lens + B_);
        pass_pending_ = true;
        worker_.submit([this, lens] { background_pass(lens); });
    }
    c_.step_us += now_us() - t_begin;
    return rc;
}

// Runs on the helper thread between a step() and the next sync().  During that window the caller's
// thread touches none of mapped_, held_, free_handles_, c_ (it validates launches against committed_),
// and active_ is read-only for both.
void KvMemory::background_pass(const std::vector<int64_t>& lens) {
    const double t0 = now_us();
    // 1. look-ahead (Sec. 6.1.1): the growth the coming iterations are known to need
    for (int r = 0; r < B_; ++r) {
        if (!active_[r] || lens[r] == 0) continue;
        const int64_t ahead = lens[r] + lookahead_ < L_ ? lens[r] + lookahead_ : L_;
        const int64_t grow = need(ahead) - mapped_[r];
        if (grow > 0 && grow * nbuf_ <= free_now()) (void)map_rows(r, mapped_[r], mapped_[r] + grow, true);
    }
    if (policy_ == VATTN_POLICY_DEFERRED) {
        const int cand = next_candidate();
        // 2. threshold reclamation (Sec. 6.1.2): inactive ids give pages back only when the pool runs low
        if (free_now() < reclaim_threshold_) {
            for (int r = 0; r < B_ && free_now() < reclaim_threshold_; ++r) {
                if (active_[r] || r == cand) continue;
                while (mapped_[r] > 0 && free_now() < reclaim_threshold_) unmap_rows(r, mapped_[r] - 1);
            }
        }
        // 3. eager allocation (Sec. 6.1.2): keep the reqId that will be handed out next backed
        if (cand >= 0 && eager_ > mapped_[cand]) {
            int64_t grow = eager_ - mapped_[cand];
            const int64_t fit = free_now() / nbuf_;
            if (grow > fit) grow = fit;
            if (grow > 0) (void)map_rows(cand, mapped_[cand], mapped_[cand] + grow, true);
        }
    }
    c_.background_us += now_us() - t0;
}

}  // namespace vattn
