// Decode attention over virtually contiguous KV: split-K kernel + reduce kernel.
//
// What is computed is Eq. 2 of the paper for one query token per request, o = softmax(q K^T * scale) V,
// with K, V read straight from the request's sub-tensor at base + reqId*S (Sec. 5.2.3) - the kernel
// never consults a block table.  The contexts of all requests, cut into 32-token tiles, form one
// global tile sequence that is split into segments, one per resident workgroup, so that the launch is a
// single round; the segment lengths follow the bandwidth each XCD draws (workgroup s runs on XCD s % 8,
// and on this chip the odd XCDs finish an equal share about 10 % later than the even ones).  Every
// (segment, KV head) pair is handled by ONE wavefront that keeps a running maximum m, a running sum l
// and an un-normalised output for the query heads of its KV head (the split-K scheme the paper cites
// as FlashDecoding); a segment that crosses a request boundary emits one partial per request.  A
// second kernel merges the partials of each request.
//
// gfx950 mapping
//  * The path is HBM-bound (8 or 7 flops per KV byte), so the design goal is a deep, fully coalesced
//    load stream: the waves of a workgroup take the KV heads of the SAME token range, so together
//    they read one contiguous byte range of K and one of V.  Every lane loads 16 bytes through a raw
//    buffer resource (scalar base + scalar tile offset + one per-lane offset); a wave has 16 such loads
//    in flight (one 32-token tile of K and of V) while it computes the previous tile.
//  * The two contractions run on the matrix cores (v_mfma_f32_16x16x32_bf16).  Scores are computed
//    transposed, S^T = K Q^T (tokens x heads), so that each lane owns one query head: the softmax
//    state is per lane, and the exponentiated scores are already in the register layout the second
//    contraction O^T = V^T P^T wants for its B operand - P never touches LDS.
//  * K and V tiles pass through a wave-private LDS region (no workgroup barrier anywhere): K rows are
//    re-read as 16-byte A operands, V is re-read with the transposing LDS load ds_read_b64_tr_b16,
//    which delivers "8 tokens of one channel" per lane as the A operand of O^T = V^T P^T.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <mutex>

#include "vattn_internal.h"

namespace vattn {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kTile = 32;          // tokens per inner iteration of a wave
constexpr int kMaxWaves = 4;       // waves (KV heads) per workgroup, and waves per CU: more concurrent streams than
                                   // this lower the bandwidth the memory system delivers (measured: 8 per CU -4 %)
constexpr float kLog2e = 1.4426950408889634f;
// Fourth dword of a gfx9-family raw buffer resource: 32-bit data format, no swizzle, no stride.
constexpr int kRsrcWord3 = 0x00020000;
constexpr int kAuxNt = 2;  // cache-policy bit "nt": streamed once, do not keep in the caches

template <int D> struct Geo {
    static constexpr int RB = D * 2;              // bytes of one head row
    static constexpr int LPR = RB / 16;           // lanes per row
    static constexpr int RPI = 64 / LPR;          // rows per load instruction
    static constexpr int NL = kTile / RPI;        // load instructions per tile (per K, per V)
    static constexpr int KSTR = RB + 16;          // LDS row stride of K (bank-conflict-free b128 reads)
    static constexpr int VSTR = RB + 32;          // LDS row stride of V (bank-conflict-free transposed reads)
    static constexpr int WAVE_LDS = kTile * (KSTR + VSTR);
};

// Maximum over the four 16-lane rows of the wave (lanes with equal l % 16), in every lane.  v_permlane16_swap
// / v_permlane32_swap exchange rows / halves of two registers inside the vector unit; a cross-lane shuffle
// would take a round trip through LDS for each of the two steps.
__device__ __forceinline__ float row_group_max(float v) {
    const unsigned b0 = __builtin_bit_cast(unsigned, v);
    const auto s16 = __builtin_amdgcn_permlane16_swap(b0, b0, false, false);     // {r0,r0,r2,r2}, {r1,r1,r3,r3}
    v = fmaxf(__builtin_bit_cast(float, s16[0]), __builtin_bit_cast(float, s16[1]));
    const unsigned b1 = __builtin_bit_cast(unsigned, v);
    const auto s32 = __builtin_amdgcn_permlane32_swap(b1, b1, false, false);     // {lo,lo}, {hi,hi}
    return fmaxf(__builtin_bit_cast(float, s32[0]), __builtin_bit_cast(float, s32[1]));
}

// INL: the index arrays are read from the kernel-argument segment (InlineMeta) instead of global memory;
// a compile-time switch so that both variants keep these uniform reads on the scalar unit.
// PAGED: the comparison variant - K/V tiles are found through a block table instead of one pointer per request.
template <int D, bool INL, bool PAGED>
__global__ __launch_bounds__(kMaxWaves * 64) void decode_splitk_kernel(DecodeArgs a, int units, int hb_per_kv, InlineMeta im) {
    using G = Geo<D>;
    auto reqid_of = [&](int r) { if constexpr (INL) return im.v[r]; else return a.reqids[r]; };
    auto kvlen_of = [&](int r) { if constexpr (INL) return im.v[a.n + r]; else return a.kv_lens[r]; };
    auto cu_of = [&](int r) { if constexpr (INL) return im.v[2 * a.n + r]; else return a.cu_tiles[r]; };
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    // the wave index is uniform within a wave: saying so keeps the KV-head arithmetic on the scalar unit
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l = threadIdx.x & 63;
    const int unit = blockIdx.y * (blockDim.x >> 6) + wave;
    if (unit >= units) return;  // no workgroup barrier is ever used, so leaving early is safe
    const int kvh = unit / hb_per_kv;
    const int hb = unit - kvh * hb_per_kv;
    const int group = a.Hq / a.H;

    // this segment's slice of the global tile sequence, and the request its first tile belongs to
    const int seg = blockIdx.x;
    const int T0 = min((seg >> 3) * a.period + a.pre[seg & 7], a.total_tiles);
    const int T1 = min((seg >> 3) * a.period + a.pre[(seg & 7) + 1], a.total_tiles);
    int lo = 0, hi = a.n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu_of(mid) <= T0) lo = mid; else hi = mid;
    }
    const int row_stride = a.row_stride;   // bytes between consecutive tokens of this layer
    char* klds = lds_raw + wave * G::WAVE_LDS;
    char* vlds = klds + kTile * G::KSTR;
    const int hl = hb * 16 + (l & 15);
    const bool head_ok = hl < group;
    const int head = kvh * group + hl;
    const float scale_log2 = a.scale * kLog2e;

  int g0 = T0;
  for (int req = lo; g0 < T1; ++req) {
    // piece = tiles [g0, g1) of request req
    const int r_first = cu_of(req);
    const int g1 = min(T1, cu_of(req + 1));
    const int kv_len = kvlen_of(req);
    const int tok0 = (g0 - r_first) * kTile;
    const int tok1 = min((g1 - r_first) * kTile, kv_len);
    // contiguous KV: one base per request (Sec. 5.2.3); paged: only the head offset, the block comes per tile
    const int64_t sub = (PAGED ? 0 : static_cast<int64_t>(reqid_of(req)) * a.S) + static_cast<int64_t>(kvh) * G::RB;
    const char* kp = a.k_base + sub;
    const char* vp = a.v_base + sub;

    // Query heads of this wave as B operands of S^T = K Q^T: lane (n = l%16, j = l/16) holds
    // Q[head n][kb*32 + j*8 .. +8].
    bf16x8 qb[D / 32];
    {
        const char* qrow = static_cast<const char*>(a.q) + (static_cast<int64_t>(req) * a.Hq + (head_ok ? head : 0)) * G::RB;
#pragma unroll
        for (int kb = 0; kb < D / 32; ++kb) {
            u32x4 raw = *reinterpret_cast<const u32x4*>(qrow + kb * 64 + (l >> 4) * 16);
            if (!head_ok) raw = u32x4{0, 0, 0, 0};
            qb[kb] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    const int ld_row = l / G::LPR;            // row inside one load instruction
    const int ld_col = (l % G::LPR) * 16;     // byte offset inside the row
    const int lane_off = ld_row * row_stride + ld_col;
    u32x4 kreg[G::NL], vreg[G::NL];
    // K and V of one tile of this (request, KV head) as raw buffer resources: the loads take one 32-bit
    // per-lane offset (the same for the whole kernel) plus a scalar offset per instruction, and the
    // 64-bit address of the tile is scalar arithmetic, so sub-tensors of any size are addressable.
    // num_records ends at the last valid row of the tile: rows past the end of the context (ragged last
    // tile) are suppressed by the hardware range check - they return zeros and touch nothing, so no
    // byte beyond what step() has mapped is read; their scores are masked below.
    auto issue_loads = [&](u32x4 (&kreg)[G::NL], u32x4 (&vreg)[G::NL], int t) {
        const int tok = tok0 + t * kTile;
        int64_t boff;
        if constexpr (PAGED) {   // block-table lookup: a tile never straddles a block (block_tokens is a multiple of the tile)
            const int blk = a.block_table[static_cast<int64_t>(req) * a.table_stride + tok / a.block_tokens];
            boff = (static_cast<int64_t>(blk) * a.block_tokens + tok % a.block_tokens) * row_stride;
        } else {
            boff = static_cast<int64_t>(tok) * row_stride;
        }
        const int nrec = (min(kv_len - tok, kTile) - 1) * row_stride + G::RB;
        const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kp + boff), 0, nrec, kRsrcWord3);
        const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vp + boff), 0, nrec, kRsrcWord3);
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int so = i * G::RPI * row_stride;
            kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(krs, lane_off, so, kAuxNt);
            vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(vrs, lane_off, so, kAuxNt);
        }
    };
    auto stage = [&](const u32x4 (&kreg)[G::NL], const u32x4 (&vreg)[G::NL]) {
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int row = i * G::RPI + ld_row;
            *reinterpret_cast<u32x4*>(klds + row * G::KSTR + ld_col) = kreg[i];
            *reinterpret_cast<u32x4*>(vlds + row * G::VSTR + ld_col) = vreg[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    float m = -INFINITY, lsum = 0.f;
    f32x4 o[D / 16];
#pragma unroll
    for (int db = 0; db < D / 16; ++db) o[db] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int t) {
        // S^T tiles: 2 x (16 tokens x 16 heads)
        f32x4 s[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            s[r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < D / 32; ++kb) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8*>(klds + (r * 16 + (l & 15)) * G::KSTR + kb * 64 + (l >> 4) * 16);
                s[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qb[kb], s[r], 0, 0, 0);
            }
        }
        // lane holds head l%16 and tokens r*16 + (l/16)*4 + i
        const int tbase = tok0 + t * kTile + (l >> 4) * 4;
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float x = s[r][i] * scale_log2;
                if (tbase + r * 16 + i >= tok1) x = -INFINITY;
                s[r][i] = x;
                mx = fmaxf(mx, x);
            }
        mx = row_group_max(mx);
        const float m_new = fmaxf(m, mx);           // finite: every tile holds at least one valid token
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        float psum = 0.f;
        bf16x8 pb;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = __builtin_amdgcn_exp2f(s[r][i] - m_new);
                psum += p;
                pb[r * 4 + i] = static_cast<__bf16>(p);
            }
        lsum = lsum * alpha + psum;
#pragma unroll
        for (int db = 0; db < D / 16; ++db) o[db] *= alpha;

        // O^T += V^T P^T : A operand = 8 tokens of one channel per lane, via transposing LDS loads
        const int vrow = (l >> 4) * 4 + ((l & 15) >> 2);
        const int vcol = (l & 3) * 8;
#pragma unroll
        for (int db = 0; db < D / 16; ++db) {
            const char* p0 = vlds + vrow * G::VSTR + db * 32 + vcol;
            const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
            const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 16 * G::VSTR));
            const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
            o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb, o[db], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    const int ntiles = g1 - g0;
    // One tile of K and V (16 loads of 16 B per lane) is in flight while the previous one is multiplied.
    // (A second register set, two tiles in flight per wave, was measured with 8, 4 and 2 waves per CU and
    // never gained: what the memory system rewards is few concurrent streams, not more bytes in flight.)
    issue_loads(kreg, vreg, 0);
    // Fused KV append (optional): the request's newest token, position kv_len - 1, has not been written to the
    // cache yet.  The one wave whose piece holds that token for this KV head puts the row into its LDS tile
    // (over whatever the cache held there) and into the cache, K by lanes 0 .. LPR-1, V by the next LPR lanes.
    const int last_local = a.k_new != nullptr && !PAGED ? kv_len - 1 - tok0 : -1;   // token index inside the piece, or out of reach
    for (int t = 0; t < ntiles; ++t) {
        stage(kreg, vreg);
        if (t + 1 < ntiles) issue_loads(kreg, vreg, t + 1);
        if (last_local >= t * kTile && last_local < (t + 1) * kTile) {   // uniform; true for at most one tile of one piece
            if (l < 2 * G::LPR) {
                const bool is_v = l >= G::LPR;
                const int c = (l % G::LPR) * 16;
                const char* src = static_cast<const char*>(is_v ? a.v_new : a.k_new) + (static_cast<int64_t>(req) * a.H + kvh) * G::RB + c;
                const u32x4 x = *reinterpret_cast<const u32x4*>(src);
                const int row = last_local - t * kTile;
                *reinterpret_cast<u32x4*>((is_v ? vlds + row * G::VSTR : klds + row * G::KSTR) + c) = x;
                *reinterpret_cast<u32x4*>(const_cast<char*>(is_v ? vp : kp) + static_cast<int64_t>(kv_len - 1) * row_stride + c) = x;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        compute(t);
    }

    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (head_ok) {
        const int64_t slot = static_cast<int64_t>(seg) + req;
        float* po = a.part_o + (slot * a.Hq + head) * D + (l >> 4) * 4;
#pragma unroll
        for (int db = 0; db < D / 16; ++db) *reinterpret_cast<f32x4*>(po + db * 16) = o[db];
        if ((l >> 4) == 0) {
            float* pml = a.part_ml + (slot * a.Hq + head) * 2;
            pml[0] = m;
            pml[1] = lsum;
        }
    }
    g0 = g1;
  }
}

// Merge of the segment partials of one (request, query head):
//   M = max_s m_s,   o = sum_s 2^(m_s-M) o_s / sum_s 2^(m_s-M) l_s.
// One workgroup of kReduceWaves waves per (request, head).  Pass 1: all threads scan the m_s for the
// maximum.  Pass 2: wave w takes chunks w, w+W, ... (lanes cover the channels, 2 per lane for
// D = 128) with independent multiply-adds, so the loads of many chunks are in flight at once; the
// wave sums are combined through LDS.
constexpr int kReduceWaves = 8;

template <int D, bool INL>
__global__ __launch_bounds__(kReduceWaves * 64) void decode_reduce_kernel(DecodeArgs a, InlineMeta im) {
    constexpr int V = D / 64;  // channels per lane
    const int req = blockIdx.x / a.Hq;
    const int head = blockIdx.x - req * a.Hq;
    // partial slots of this request: the segments of its first .. last tile, + req
    int t_first, t_end;
    if constexpr (INL) { t_first = im.v[2 * a.n + req]; t_end = im.v[2 * a.n + req + 1]; }
    else { t_first = a.cu_tiles[req]; t_end = a.cu_tiles[req + 1]; }
    auto seg_of = [&](int t) {   // the segment that holds tile t
        const int p = t / a.period, r = t - p * a.period;
        int x = 0;
#pragma unroll
        for (int i = 1; i < 8; ++i) x += r >= a.pre[i];
        return p * 8 + x;
    };
    const int c0 = seg_of(t_first) + req;
    const int c1 = seg_of(t_end - 1) + req + 1;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    __shared__ float sh_max[kReduceWaves];
    __shared__ float sh_acc[kReduceWaves][D];
    __shared__ float sh_den[kReduceWaves];

    float M = -INFINITY;
    for (int c = c0 + static_cast<int>(threadIdx.x); c < c1; c += kReduceWaves * 64)
        M = fmaxf(M, a.part_ml[(static_cast<int64_t>(c) * a.Hq + head) * 2]);
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) M = fmaxf(M, __shfl_xor(M, sft));
    if (l == 0) sh_max[w] = M;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kReduceWaves; ++i) M = fmaxf(M, sh_max[i]);   // finite: c1 > c0 always

    float den = 0.f, acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
#pragma unroll 4
    for (int c = c0 + w; c < c1; c += kReduceWaves) {
        const int64_t idx = static_cast<int64_t>(c) * a.Hq + head;
        const float f = __builtin_amdgcn_exp2f(a.part_ml[idx * 2] - M);
        den += f * a.part_ml[idx * 2 + 1];
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += f * a.part_o[idx * D + l * V + e];
    }
#pragma unroll
    for (int e = 0; e < V; ++e) sh_acc[w][l * V + e] = acc[e];
    if (l == 0) sh_den[w] = den;
    __syncthreads();
    if (w == 0) {
        float dt = 0.f, out[V];
#pragma unroll
        for (int e = 0; e < V; ++e) out[e] = 0.f;
#pragma unroll
        for (int i = 0; i < kReduceWaves; ++i) {
            dt += sh_den[i];
#pragma unroll
            for (int e = 0; e < V; ++e) out[e] += sh_acc[i][l * V + e];
        }
        __bf16* dst = static_cast<__bf16*>(a.o) + (static_cast<int64_t>(req) * a.Hq + head) * D + l * V;
        const float inv = 1.f / dt;
#pragma unroll
        for (int e = 0; e < V; ++e) dst[e] = static_cast<__bf16>(out[e] * inv);
    }
}

// The same merge for requests that own few partials (a batch of many requests, the usual decode case): one
// wave per (request, query head), four per workgroup, no LDS and no barrier - the lanes first share the
// maximum, then walk the partials with independent multiply-adds.  An eighth of the waves of the kernel above.
constexpr int kReduceFewPairs = 4;

template <int D, bool INL>
__global__ __launch_bounds__(kReduceFewPairs * 64) void decode_reduce_few_kernel(DecodeArgs a, InlineMeta im) {
    constexpr int V = D / 64;  // channels per lane
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
    const int pair = blockIdx.x * kReduceFewPairs + w;
    if (pair >= a.n * a.Hq) return;
    const int req = pair / a.Hq;
    const int head = pair - req * a.Hq;
    int t_first, t_end;
    if constexpr (INL) { t_first = im.v[2 * a.n + req]; t_end = im.v[2 * a.n + req + 1]; }
    else { t_first = a.cu_tiles[req]; t_end = a.cu_tiles[req + 1]; }
    auto seg_of = [&](int t) {   // the segment that holds tile t
        const int p = t / a.period, r = t - p * a.period;
        int x = 0;
#pragma unroll
        for (int i = 1; i < 8; ++i) x += r >= a.pre[i];
        return p * 8 + x;
    };
    const int c0 = seg_of(t_first) + req;
    const int c1 = seg_of(t_end - 1) + req + 1;

    float M = -INFINITY;
    for (int c = c0 + l; c < c1; c += 64) M = fmaxf(M, a.part_ml[(static_cast<int64_t>(c) * a.Hq + head) * 2]);
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) M = fmaxf(M, __shfl_xor(M, sft));   // finite: c1 > c0 always

    float den = 0.f, acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
#pragma unroll 4
    for (int c = c0; c < c1; ++c) {
        const int64_t idx = static_cast<int64_t>(c) * a.Hq + head;
        const float f = __builtin_amdgcn_exp2f(a.part_ml[idx * 2] - M);
        den += f * a.part_ml[idx * 2 + 1];
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += f * a.part_o[idx * D + l * V + e];
    }
    __bf16* dst = static_cast<__bf16*>(a.o) + (static_cast<int64_t>(req) * a.Hq + head) * D + l * V;
    const float inv = 1.f / den;
#pragma unroll
    for (int e = 0; e < V; ++e) dst[e] = static_cast<__bf16>(acc[e] * inv);
}

}  // namespace

static const InlineMeta kNoInline{};

// Split-K partials for callers that cannot allocate (vattn_attn_decode_static): a device array the library
// itself owns, one copy per GPU, held until the process ends.  In host code the array's name is only a
// stand-in; its device address is asked of the runtime once per device and kept.
static __device__ __align__(256) unsigned char scratch[kDecodeScratchBytes];

bool decode_static_scratch(int device, void** ptr, size_t* bytes) {
    constexpr int kMaxDevices = 64;
    static void* addr[kMaxDevices] = {};
    static std::mutex mu;                       // contexts on different threads may ask at the same time
    if (device < 0 || device >= kMaxDevices) { set_error("attn_decode_static: device ordinal out of range"); return false; }
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[device]) {
        int current = -1;
        if (!hip_ok(hipGetDevice(&current), "hipGetDevice")) return false;
        if (current != device && !hip_ok(hipSetDevice(device), "hipSetDevice")) return false;
        void* p = nullptr;
        const bool ok = hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress (decode scratch)");
        if (current != device && current >= 0) (void)hipSetDevice(current);
        if (!ok || !p) { if (ok) set_error("attn_decode_static: the runtime returned no address for the scratch array"); return false; }
        addr[device] = p;
    }
    *ptr = addr[device];
    *bytes = kDecodeScratchBytes;
    return true;
}

static int waves_per_workgroup(int Hq, int H) {
    const int units = H * ((Hq / H + 15) / 16);
    return units < kMaxWaves ? units : kMaxWaves;
}

// A CU is given kMaxWaves waves of this kernel.
int decode_resident_workgroups(int Hq, int H, int D, int num_cus) {
    (void)D;
    const int units = H * ((Hq / H + 15) / 16);
    const int waves = waves_per_workgroup(Hq, H);
    const int wg_per_cu = kMaxWaves / waves;
    const int ygrid = (units + waves - 1) / waves;
    const int segs = num_cus * wg_per_cu / ygrid;
    return segs > 0 ? segs : 1;
}

bool launch_decode_splitk(const DecodeArgs& a, const InlineMeta* im, hipStream_t stream, LaunchEvents ev) {
    const InlineMeta& meta = im ? *im : kNoInline;
    const int group = a.Hq / a.H;
    const int hb_per_kv = (group + 15) / 16;
    const int units = a.H * hb_per_kv;
    const int waves = waves_per_workgroup(a.Hq, a.H);
    // Workgroups are dealt to the XCDs in launch order, x fastest: with several workgroups per segment (grid.y)
    // the x extent is padded to a multiple of 8 so that segment s still lands on XCD s % 8 in every row; the
    // padding segments are empty.
    const unsigned ygrid = static_cast<unsigned>((units + waves - 1) / waves);
    const unsigned xgrid = ygrid > 1 ? (static_cast<unsigned>(a.num_segs) + 7u) / 8u * 8u : static_cast<unsigned>(a.num_segs);
    dim3 grid(xgrid, ygrid);
    dim3 block(static_cast<unsigned>(waves * 64));
    static bool allowed[8] = {};  // per kernel variant
    auto launch = [&](auto kernel, size_t wave_lds, int variant) -> bool {
        // dynamic LDS above 64 KiB has to be allowed once per kernel
        if (!allowed[variant]) {
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kMaxWaves * wave_lds)), "hipFuncSetAttribute")) return false;
            allowed[variant] = true;
        }
        hipExtLaunchKernelGGL(kernel, grid, block, static_cast<size_t>(waves) * wave_lds, stream, ev.start, ev.stop, 0, a, units, hb_per_kv, meta);
        return true;
    };
    bool ok;
    if (a.block_table) {
        if (a.D == 128) ok = a.inline_meta ? launch(decode_splitk_kernel<128, true, true>, Geo<128>::WAVE_LDS, 4) : launch(decode_splitk_kernel<128, false, true>, Geo<128>::WAVE_LDS, 5);
        else ok = a.inline_meta ? launch(decode_splitk_kernel<64, true, true>, Geo<64>::WAVE_LDS, 6) : launch(decode_splitk_kernel<64, false, true>, Geo<64>::WAVE_LDS, 7);
    } else {
        if (a.D == 128) ok = a.inline_meta ? launch(decode_splitk_kernel<128, true, false>, Geo<128>::WAVE_LDS, 0) : launch(decode_splitk_kernel<128, false, false>, Geo<128>::WAVE_LDS, 1);
        else ok = a.inline_meta ? launch(decode_splitk_kernel<64, true, false>, Geo<64>::WAVE_LDS, 2) : launch(decode_splitk_kernel<64, false, false>, Geo<64>::WAVE_LDS, 3);
    }
    if (!ok) return false;
    return hip_ok(hipGetLastError(), "decode split-K launch");
}

bool launch_decode_reduce(const DecodeArgs& a, const InlineMeta* im, hipStream_t stream, LaunchEvents ev) {
    const InlineMeta& meta = im ? *im : kNoInline;
    if (a.max_slots <= 16) {   // few partials per request: one wave per (request, head)
        const dim3 grid(static_cast<unsigned>((a.n * a.Hq + kReduceFewPairs - 1) / kReduceFewPairs));
        const dim3 block(kReduceFewPairs * 64);
        if (a.D == 128) {
            if (a.inline_meta) hipExtLaunchKernelGGL((decode_reduce_few_kernel<128, true>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
            else hipExtLaunchKernelGGL((decode_reduce_few_kernel<128, false>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
        } else {
            if (a.inline_meta) hipExtLaunchKernelGGL((decode_reduce_few_kernel<64, true>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
            else hipExtLaunchKernelGGL((decode_reduce_few_kernel<64, false>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
        }
        return hip_ok(hipGetLastError(), "decode reduce launch");
    }
    dim3 grid(static_cast<unsigned>(a.n * a.Hq));
    const dim3 block(kReduceWaves * 64);
    if (a.D == 128) {
        if (a.inline_meta) hipExtLaunchKernelGGL((decode_reduce_kernel<128, true>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
        else hipExtLaunchKernelGGL((decode_reduce_kernel<128, false>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
    } else {
        if (a.inline_meta) hipExtLaunchKernelGGL((decode_reduce_kernel<64, true>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
        else hipExtLaunchKernelGGL((decode_reduce_kernel<64, false>), grid, block, 0, stream, ev.start, ev.stop, 0, a, meta);
    }
    return hip_ok(hipGetLastError(), "decode reduce launch");
}

}  // namespace vattn
