// Split-K plan of the decode path: how the batch's 32-token tiles are cut into segments.  Pure host
// arithmetic without any GPU call, so that it can be built and checked on a machine without a GPU; the
// kernels (attn_decode.hip) recompute a segment's range and a tile's segment from the same nine numbers.
//
// The tiles of all requests form one sequence (request-major).  It is cut into as many segments as one
// launch keeps resident on the chip - or into segments of a fixed tile count when the caller set a chunk
// size.  Workgroup s of a launch runs on XCD s % 8 and the XCDs do not draw the same bandwidth, so the
// segment lengths repeat with period 8 and follow eight weights; the last period may be cut short by the
// end of the sequence.  Segment s owns tiles [(s/8)*period + pre[s%8], (s/8)*period + pre[s%8 + 1]),
// clipped to the sequence.  Inside the sequence no segment is empty (only the grid's padding segments
// past num_segs are).
#pragma once

#include <algorithm>
#include <cstdint>

namespace vattn {

struct DecodePlan {
    int64_t total_tiles;
    int num_segs;      // segments 0 .. num_segs-1 cover the sequence; later ones would be empty
    int period;        // tiles per group of 8 segments
    int pre[9];        // pre[0] = 0 <= pre[1] <= ... <= pre[8] = period
};

// chunk_tokens: 0 = one segment per resident workgroup slot (times segments_per_slot), else the fixed segment
// length in tokens (a multiple of 32).  weights: 8 positive numbers.
inline DecodePlan make_decode_plan(const int64_t* kv_lens, int n, int chunk_tokens, int resident_workgroups,
                                   int segments_per_slot, const float* weights) {
    DecodePlan p{};
    for (int i = 0; i < n; ++i) p.total_tiles += (kv_lens[i] + 31) / 32;
    int64_t len[8];
    if (chunk_tokens > 0) {
        for (int x = 0; x < 8; ++x) len[x] = chunk_tokens / 32;
    } else {
        const int64_t segs = std::max<int64_t>(8, static_cast<int64_t>(resident_workgroups) * segments_per_slot / 8 * 8);
        const int64_t periods = segs / 8;
        const int64_t P = (p.total_tiles + periods - 1) / periods;     // tiles per period
        if (P < 64) {   // short contexts: equal segments, as many as there are tiles if need be
            const int64_t tps = std::max<int64_t>(1, (p.total_tiles + segs - 1) / segs);
            for (int x = 0; x < 8; ++x) len[x] = tps;
        } else {        // weighted lengths that add up to P (largest remainders get the leftover tiles)
            double wsum = 0;
            for (int x = 0; x < 8; ++x) wsum += weights[x];
            double frac[8];
            int64_t used = 0;
            for (int x = 0; x < 8; ++x) {
                const double exact = static_cast<double>(P) * weights[x] / wsum;
                len[x] = static_cast<int64_t>(exact);
                frac[x] = exact - static_cast<double>(len[x]);
                used += len[x];
            }
            for (; used < P; ++used) {
                int best = 0;
                for (int x = 1; x < 8; ++x) if (frac[x] > frac[best]) best = x;
                ++len[best]; frac[best] = -1;
            }
            // No segment of a full period may be empty: the reduce kernel reads every partial slot between a
            // request's first and last segment, and an empty segment writes none.  A weight small enough to
            // round to zero tiles takes one from the longest segment instead (P >= 64, so that one stays long).
            for (int x = 0; x < 8; ++x) {
                if (len[x] > 0) continue;
                int longest = 0;
                for (int y = 1; y < 8; ++y) if (len[y] > len[longest]) longest = y;
                --len[longest]; ++len[x];
            }
        }
    }
    int64_t acc = 0;
    for (int x = 0; x < 8; ++x) { p.pre[x] = static_cast<int>(acc); acc += len[x]; }
    p.pre[8] = static_cast<int>(acc);
    p.period = p.pre[8];
    const int64_t full = p.total_tiles / p.period, rest = p.total_tiles % p.period;
    int tail = 0;
    while (tail < 8 && p.pre[tail] < rest) ++tail;     // segments of the last, partial period that hold tiles
    p.num_segs = static_cast<int>(std::max<int64_t>(1, full * 8 + tail));
    return p;
}

// Upper bound of num_segs over all batches in the default mode (chunk_tokens = 0), for sizing a workspace once.
inline int decode_plan_max_segs(int resident_workgroups, int segments_per_slot) {
    return std::max(8, resident_workgroups * segments_per_slot) + 8;
}

// The segment that holds tile t (what the reduce kernel computes).
inline int64_t decode_plan_segment_of(const DecodePlan& p, int64_t t) {
    const int64_t q = t / p.period, r = t % p.period;
    int x = 0;
    for (int i = 1; i < 8; ++i) x += r >= p.pre[i];
    return q * 8 + x;
}

}  // namespace vattn
