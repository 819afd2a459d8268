// Host build of the decode split-K planner (csrc/decode_plan.h).  Reads one request per line:
//   chunk_tokens resident segments_per_slot w0 .. w7 len0 len1 ...
// and prints: total_tiles num_segs max_segs period pre0 .. pre8
#include <cstdio>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../../paper_2405_04437_amd/csrc/decode_plan.h"

int main() {
    std::string line;
    while (std::getline(std::cin, line)) {
        std::istringstream in(line);
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
