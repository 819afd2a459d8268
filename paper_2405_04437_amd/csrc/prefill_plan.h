// Work queues of the prefill path.  Pure host arithmetic without any GPU call, so that it can be built and
// checked on a machine without a GPU.
//
// A work item is one (request, KV head, query tile of BM rows); the kernel runs it once per query head of
// the KV head's group.  There is one queue per XCD: workgroup ids are dealt to the 8 XCDs round-robin, so
// giving XCD x the streams (request, KV head, tile class) with index == x (mod 8) keeps all readers of one
// K/V stream behind the same L2.  KV heads are split into tile classes when there are fewer than 8.  Every
// queue is sorted by cost (keys the tile can see), longest first, and padded with req = -1 to a common length.
#pragma once

#include <algorithm>
#include <cstdint>
#include <vector>

namespace vattn {

// What a workgroup needs to start on a work item, in one 32-byte record (one scalar load): the batch slot, the
// KV head, the query tile, and the request's reqId, first query row, chunk length and context length.
struct PrefillItem { int32_t req; int32_t kvh; int32_t q_tile; int32_t reqid; int32_t q_begin; int32_t q_len; int32_t kv_len; int32_t pad; };

struct PrefillQueues {
    int waves;                        // waves per workgroup (8 or 12)
    int rows_per_item;                // BM: 32 * waves
    int per_xcd;                      // entries per queue, padding included
    std::vector<PrefillItem> items;   // 8 * per_xcd entries, queue x at [x * per_xcd, (x + 1) * per_xcd)
};

// Twelve waves (384 rows per work item, three waves per SIMD) when that still leaves every CU several work
// items, else eight waves (256 rows).
// reqids may be null (paged comparison variant: the record then carries 0).
inline PrefillQueues make_prefill_queues(const int32_t* reqids, const int32_t* cu_q, const int64_t* kv_lens, int n, int Hq, int H, int num_cus) {
    PrefillQueues out{};
    out.waves = 8;
    int64_t items12 = 0;
    for (int r = 0; r < n; ++r) items12 += (static_cast<int64_t>(cu_q[r + 1]) - cu_q[r] + 383) / 384 * Hq;
    if (items12 >= 4 * static_cast<int64_t>(num_cus)) out.waves = 12;
    const int BM = 32 * out.waves;
    out.rows_per_item = BM;
    const int nsplit = H < 8 ? (8 + H - 1) / H : 1;
    struct Cost { PrefillItem it; int64_t cost; };
    std::vector<Cost> queues[8];
    for (int r = 0; r < n; ++r) {
        const int ql = cu_q[r + 1] - cu_q[r];
        const int tiles = (ql + BM - 1) / BM;
        const int64_t off = kv_lens[r] - ql;
        for (int t = 0; t < tiles; ++t) {
            const int64_t visible = std::min<int64_t>(static_cast<int64_t>(t + 1) * BM, ql) + off;
            for (int kvh = 0; kvh < H; ++kvh) {
                const int x = (kvh * nsplit + t % nsplit + ((H * nsplit) % 8 ? r : 0)) & 7;
                queues[x].push_back(Cost{PrefillItem{r, kvh, t, reqids ? reqids[r] : 0, cu_q[r], ql, static_cast<int32_t>(kv_lens[r]), 0}, visible});
            }
        }
    }
    size_t per_xcd = 0;
    for (auto& qx : queues) {
        std::stable_sort(qx.begin(), qx.end(), [](const Cost& x, const Cost& y) { return x.cost > y.cost; });
        per_xcd = std::max(per_xcd, qx.size());
    }
    out.per_xcd = static_cast<int>(per_xcd);
    out.items.assign(per_xcd * 8, PrefillItem{-1, 0, 0, 0, 0, 0, 0, 0});
    for (int x = 0; x < 8; ++x)
        for (size_t j = 0; j < queues[x].size(); ++j) out.items[x * per_xcd + j] = queues[x][j].it;
    return out;
}

}  // namespace vattn
