// Host build of the launch planners (csrc/decode_plan.h, csrc/prefill_plan.h).  One request per line:
//   chunk_tokens resident segments_per_slot w0 .. w7 len0 len1 ...
//       -> total_tiles num_segs max_segs period pre0 .. pre8
//   Q Hq H num_cus n q_len0 kv_len0 q_len1 kv_len1 ...
//       -> waves rows_per_item per_xcd, then 8 * per_xcd records req kvh q_tile reqid q_begin q_len kv_len (queue-major;
//          batch slot r is given reqId 1000 + 7 r)
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../../paper_2405_04437_amd/csrc/decode_plan.h"
#include "../../paper_2405_04437_amd/csrc/prefill_plan.h"

int main() {
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
        if (!line.empty() && line[0] == 'Q') {
            char tag;
            int Hq, H, cus, n;
            in >> tag >> Hq >> H >> cus >> n;
            std::vector<int32_t> cu(1, 0);
            std::vector<int64_t> kv;
            for (int r = 0; r < n; ++r) { int q; long long k; in >> q >> k; cu.push_back(cu.back() + q); kv.push_back(k); }
            std::vector<int32_t> ids;
            for (int r = 0; r < n; ++r) ids.push_back(1000 + 7 * r);   // reqIds the records must carry
            const vattn::PrefillQueues pq = vattn::make_prefill_queues(ids.data(), cu.data(), kv.data(), n, Hq, H, cus);
            std::printf("%d %d %d", pq.waves, pq.rows_per_item, pq.per_xcd);
            for (const auto& it : pq.items) std::printf(" %d %d %d %d %d %d %d", it.req, it.kvh, it.q_tile, it.reqid, it.q_begin, it.q_len, it.kv_len);
            std::printf("\n");
            std::fflush(stdout);
            continue;
        }
        int chunk, resident, per_slot;
        float w[8];
        if (!(in >> chunk >> resident >> per_slot)) break;
        for (float& x : w) in >> x;
        std::vector<int64_t> lens;
        long long v;
        while (in >> v) lens.push_back(v);
        const vattn::DecodePlan p = vattn::make_decode_plan(lens.data(), static_cast<int>(lens.size()), chunk, resident, per_slot, w);
        std::printf("%lld %d %d %d", static_cast<long long>(p.total_tiles), p.num_segs, vattn::decode_plan_max_segs(resident, per_slot), p.period);
        for (int x = 0; x < 9; ++x) std::printf(" %d", p.pre[x]);
        std::printf("\n");
        std::fflush(stdout);
    }
    return 0;
}
