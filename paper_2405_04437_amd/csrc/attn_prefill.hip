// Causal prefill attention over virtually contiguous KV.
//
// Computes Eq. 2 of the paper per request, o_i = softmax(q_i K^T * scale) V over the keys visible to
// query row i (keys 0 .. kv_len - q_len + i), with K and V read in place from the request's
// sub-tensor at base + reqId*S (Sec. 5.2.3): no block table, one pointer and one stride.
//
// gfx950 mapping
//  * One workgroup per CU: 8 waves (two per SIMD, 256 query rows of one query head) or, when the launch
//    has enough work items to keep every CU busy for several rounds, 12 waves (three per SIMD, 384 rows);
//    32 rows per wave, all waves share each K/V tile.  KV is walked in tiles
//    of 64 tokens through a four-stage LDS ring, two tiles per workgroup barrier; tiles travel from
//    global memory straight into LDS (buffer loads with the LDS bit) two tiles ahead of their use.
//  * Both contractions use v_mfma_f32_32x32x16_bf16.  Scores are produced transposed,
//    S^T = K Q^T (tokens x rows): a lane then owns ONE query row, so the running max / sum are
//    per-lane scalars (one cross-lane exchange per tile), and exp(S^T) is already laid out as the B
//    operand of O^T = V^T P^T.  V^T comes out of LDS through ds_read_b64_tr_b16.
//  * The launch is XCD-aware: workgroup ids are dealt round-robin to the 8 XCDs by the hardware, so
//    the host builds one work queue per XCD and gives each XCD whole (request, KV head) streams; the
//    query heads of a group and neighbouring query tiles then run on the same XCD at the same time
//    and share the K/V stream through that XCD's L2.
//  * Workgroups are persistent: one per CU, each takes the next slot of its XCD's queue from an atomic
//    counter and, once that queue is drained, helps with the queues of the other XCDs (the XCDs do not
//    run at the same speed).  Starting a new workgroup per work item instead left each CU idle for about
//    10 us per item.
//  * Optional fused KV append (template flag FUSED): the chunk's own K/V rows are read from the caller's
//    arrays and stored into the cache by the same launch (what Sec. 7.1 of the paper does with a copy).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "vattn_internal.h"

namespace vattn {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kBN = 64;    // KV tokens per tile
constexpr float kLog2e = 1.4426950408889634f;
// The running maximum is only raised when some row's tile maximum exceeds it by more than this many
// binary orders of magnitude: exponentials then stay below 2^kLazy, which fp32 sums and bf16 P hold
// easily, and the O accumulator is rescaled a handful of times per row instead of once per tile.
constexpr float kLazy = 8.0f;
// Fourth dword of a gfx9-family raw buffer resource: 32-bit data format, no swizzle, no stride.
constexpr int kRsrcWord3 = 0x00020000;

// D: head dimension; NW: waves per workgroup (8 or 12), 32 query rows each.
template <int D, int NW> struct PGeo {
    static constexpr int RB = D * 2;                         // bytes per head row
    static constexpr int CH = RB / 16;                       // 16-byte chunks per row
    static constexpr int RPW = 1024 / RB;                    // rows one wave-wide 16 B/lane load covers
    static constexpr int NB = kBN / RPW;                     // such loads per tile and tensor; wave w issues loads w, w+NW, ...
    static constexpr int NLW = (NB + NW - 1) / NW;           // at most this many per wave
    static constexpr int KV = kBN * RB;                      // one K (or V) tile in LDS, rows unpadded
    static constexpr int BUF = 2 * KV;                       // one K+V stage
    static constexpr int STAGES = 4;                         // two tiles being read, two arriving
    static constexpr int LDS = STAGES * BUF;
    // Rows are stored unpadded (the loads below write LDS directly, 1 KiB contiguous per instruction), so
    // bank conflicts are avoided by permuting the 16-byte chunks inside each row instead: chunk c of row r
    // is stored at chunk position c ^ swz(r).  LDS has 64 banks of 4 bytes, i.e. 256 bytes per clock:
    //  * a K fragment read (16 B per lane) is served 16 lanes at a time - 16 consecutive rows, same logical
    //    chunk - so the K permutation takes 16 different values over 16 rows' worth of 256 B;
    //  * a transposing V read (8 B per lane) is served 32 lanes at a time - 4 consecutive rows, 64 B each -
    //    so the V permutation moves whole 64-byte groups (4 chunks) and differs between those 4 rows.
    __device__ static constexpr int swz_k(int row) { return (row * RB / 256) & (CH - 1); }
    __device__ static constexpr int swz_v(int row) { return ((row * RB / 256) & (RB / 64 - 1)) << 2; }
};

typedef __attribute__((address_space(3))) void* lds_ptr;

// FUSED: the K/V rows of the query tokens arrive in a.k_new / a.v_new and are not in the cache yet.  Tiles at or
// beyond position kv_len - q_len are read from those arrays (rows H*D apart), and the first
// query head of every group stores the rows of its query tile into the cache; no workgroup ever reads a cache
// row that this launch writes.
template <int D, int NW, bool FUSED>
__global__ __launch_bounds__(NW * 64, NW / 4) void prefill_kernel(PrefillArgs a) {
    using G = PGeo<D, NW>;
    constexpr int kWaves = NW;
    // matrix operands are requested from LDS this many multiplies ahead; three waves per SIMD leave 168
    // registers per lane, which a depth of 6 does not fit
    constexpr int kAhead = NW > 8 ? 4 : 6;
    constexpr int BM = NW * 32;                // query rows per workgroup
    constexpr int WR = 32;                     // query rows per wave
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform per wave: keeps row/tile arithmetic scalar
    const int l = tid & 63;
    const int group = a.Hq / a.H;

    // persistent workgroup: takes the next slot of its XCD's queue; when that is drained, of the others
    __shared__ int sh_item[2];
    const int cap = a.items_per_xcd * group;
    int xcd = blockIdx.x & 7;
  for (;;) {
    if (tid == 0) {
        int got = -1, from = xcd;
        for (int tries = 0; tries < 8 && got < 0; ++tries) {
            const int x = (xcd + tries) & 7;
            if (__hip_atomic_load(&a.queue_heads[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < cap) {
                const int s2 = atomicAdd(&a.queue_heads[x], 1);
                if (s2 < cap && a.items[static_cast<int64_t>(x) * a.items_per_xcd + s2 / group].req >= 0) { got = s2; from = x; }
            }
        }
        sh_item[0] = got; sh_item[1] = from;
    }
    __syncthreads();
    const int slot = __builtin_amdgcn_readfirstlane(sh_item[0]);
    xcd = __builtin_amdgcn_readfirstlane(sh_item[1]);
    if (slot < 0) return;
    const PrefillItem it = a.items[static_cast<int64_t>(xcd) * a.items_per_xcd + slot / group];
    const int head = it.kvh * group + slot % group;
    const int req = it.req;
    const int q_begin = it.q_begin;
    const int q_len = it.q_len;
    const int kv_len = it.kv_len;
    const int off = kv_len - q_len;            // query row i sees keys 0 .. i + off
    const int q0 = it.q_tile * BM;
    const int q_last = min(q0 + BM, q_len) - 1;
    const int n_kv = q_last + off + 1;         // keys any row of this tile can see
    const int ntiles = (n_kv + kBN - 1) / kBN;

    const int rs32 = a.row_stride;             // bytes between consecutive tokens of this layer
    // contiguous KV: one base per request; paged comparison variant: only the head offset, the block comes per tile
    const bool paged = a.block_table != nullptr;
    const int64_t sub = (paged ? 0 : static_cast<int64_t>(it.reqid) * a.S) + static_cast<int64_t>(it.kvh) * G::RB;
    const char* kp = a.k_base + sub;
    const char* vp = a.v_base + sub;
    const char* kn = nullptr;
    const char* vn = nullptr;
    // bytes between consecutive new rows [.., H, D]: the cache's own token stride unless all layers share a buffer
    const int ns32 = FUSED ? a.H * G::RB : rs32;
    if constexpr (FUSED) {
        // row j of the request's new rows is position off + j of its context
        const int64_t nsub = (static_cast<int64_t>(q_begin) * a.H + it.kvh) * G::RB;
        kn = static_cast<const char*>(a.k_new) + nsub;
        vn = static_cast<const char*>(a.v_new) + nsub;
        if (slot % group == 0) {   // one query head per (request, KV head, query tile) stores that tile's rows
            const int nrows = min(q0 + BM, q_len) - q0;
            for (int i = tid; i < nrows * G::CH; i += NW * 64) {
                const int row = q0 + i / G::CH, c = (i % G::CH) * 16;
                const int64_t src = static_cast<int64_t>(row) * ns32 + c;
                const int64_t dst = static_cast<int64_t>(off + row) * rs32 + c;
                const u32x4 kx = *reinterpret_cast<const u32x4*>(kn + src);
                const u32x4 vx = *reinterpret_cast<const u32x4*>(vn + src);
                *reinterpret_cast<u32x4*>(const_cast<char*>(kp) + dst) = kx;
                *reinterpret_cast<u32x4*>(const_cast<char*>(vp) + dst) = vx;
            }
        }
    }

    // Q^T as B operand: lane (n = l%32, h = l/32) holds Q[row n][ks*16 + h*8 .. +8]
    const int row_lo = q0 + w * WR;               // first query row of this wave
    const int my_row = row_lo + (l & 31);
    bf16x8 qb[D / 16];
    {
        const int qr = min(my_row, q_len - 1);
        const char* qrow = static_cast<const char*>(a.q) + ((static_cast<int64_t>(q_begin) + qr) * a.Hq + head) * G::RB;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qb[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + ks * 32 + (l >> 5) * 16));
    }

    // K/V tiles go from global memory straight into LDS (buffer loads with the LDS bit): no staging
    // registers, no LDS store instructions.  One wave-wide load moves 64 x 16 B = RPW whole rows into 1 KiB
    // of contiguous LDS; wave w issues loads w, w + kWaves, ... of a tile (load b carries rows b*RPW ..).  Each tile of K and V
    // is a raw buffer resource whose 64-bit base is scalar arithmetic (sub-tensors of any size are
    // addressable); a lane adds one offset that is the same for the whole kernel - its row inside the
    // load and the chunk it fetches, which is the chunk its LDS position holds under the permutation - and
    // the load adds a scalar row offset.  num_records ends at the last row of the context: rows past it
    // fail the hardware range check, touch nothing and put zeros into LDS, so no byte beyond what step()
    // has mapped is read (their scores are masked, their zero V rows are multiplied by zero weights).
    const int dma_row = l / G::CH;                                    // row inside one load
    // The chunk a lane fetches depends on the row's position in the tile: for V only on the row inside the
    // load, for K on the load's index modulo PB (the K permutation repeats every 16 rows' worth of 256 B).
    // With kWaves = 6 the loads of one wave alternate between two such positions.
    constexpr int PB = 16 * 256 / G::RB / G::RPW;                      // loads per K permutation period (4 or 2)
    constexpr int STEP = (kWaves % PB == 0) ? PB : (kWaves % PB);    // a wave's loads sit at w + multiples of STEP (mod PB)
    static_assert(PB % STEP == 0 && PB / STEP <= 2, "unsupported number of waves");
    int dma_voff_k[2];
#pragma unroll
    for (int v = 0; v < 2; ++v)
        dma_voff_k[v] = dma_row * rs32 + (((l % G::CH) ^ G::swz_k((w + v * STEP) * G::RPW + dma_row)) << 4);
    const int dma_voff_v = dma_row * rs32 + (((l % G::CH) ^ G::swz_v(dma_row)) << 4);
    // (FUSED) the new rows may lie closer together than the cache's tokens: a lane's row offset then shrinks by this much
    const int dma_row_excess = dma_row * (rs32 - ns32);
    // The loads are written as inline assembly: the compiler does not see them, so its wait-counter pass
    // does not make the LDS reads of tile t wait for the loads of tile t+1 (it cannot tell the two stages
    // apart); the waits that are needed are placed by hand before the barriers.  No other vector-memory
    // instruction is issued between the first of these loads and the end of the loop.
    const char* const kp_cache = kp;
    const char* const vp_cache = vp;
    auto issue_loads = [&](int t) {
        const int tok = t * kBN;
        const int rows = min(kv_len - tok, kBN);   // <= 0 past the end: everything out of range
        const uint32_t kb = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds)) + (t & (G::STAGES - 1)) * G::BUF;   // LDS byte address
        bool straddle = false;   // cache rows up to position off - 1, new rows from there on, in one tile
        if constexpr (FUSED) {
            if (tok >= off) {
                // A tile of new rows: same loads from the caller's arrays, whose rows are ns32 bytes apart.
                const uint32_t nrec = rows > 0 ? static_cast<uint32_t>((rows - 1) * ns32 + G::RB) : 0u;
                const uint64_t ka = reinterpret_cast<uint64_t>(kn) + static_cast<int64_t>(tok - off) * ns32;
                const uint64_t va = reinterpret_cast<uint64_t>(vn) + static_cast<int64_t>(tok - off) * ns32;
                const u32x4 krs = {static_cast<uint32_t>(ka), static_cast<uint32_t>(ka >> 32) & 0xFFFFu, nrec, static_cast<uint32_t>(kRsrcWord3)};
                const u32x4 vrs = {static_cast<uint32_t>(va), static_cast<uint32_t>(va >> 32) & 0xFFFFu, nrec, static_cast<uint32_t>(kRsrcWord3)};
#pragma unroll
                for (int j = 0; j < G::NLW; ++j) {
                    const int b = w + j * kWaves;
                    if (b < G::NB) {
                        const int so = b * G::RPW * ns32;
                        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                                     :: "s"(kb + b * 1024), "v"(dma_voff_k[((j * kWaves) % PB) / STEP] - dma_row_excess), "s"(krs), "s"(so) : "memory", "m0");
                        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                                     :: "s"(kb + G::KV + b * 1024), "v"(dma_voff_v - dma_row_excess), "s"(vrs), "s"(so) : "memory", "m0");
                    }
                }
                return;
            }
            straddle = tok + kBN > off;
        }
        int64_t boff = static_cast<int64_t>(tok) * rs32;
        if (paged && rows > 0) {   // block-table lookup; a tile never straddles a block (block_tokens is a multiple of the tile)
            const int blk = a.block_table[static_cast<int64_t>(req) * a.table_stride + tok / a.block_tokens];
            boff = (static_cast<int64_t>(blk) * a.block_tokens + tok % a.block_tokens) * rs32;
        }
        const uint32_t nrec = rows > 0 ? static_cast<uint32_t>((rows - 1) * rs32 + G::RB) : 0u;
        const uint64_t ka = reinterpret_cast<uint64_t>(kp_cache + boff), va = reinterpret_cast<uint64_t>(vp_cache + boff);
        // raw buffer resource: base[47:0], stride 0, num_records, data format word
        const u32x4 krs = {static_cast<uint32_t>(ka), static_cast<uint32_t>(ka >> 32) & 0xFFFFu, nrec, static_cast<uint32_t>(kRsrcWord3)};
        const u32x4 vrs = {static_cast<uint32_t>(va), static_cast<uint32_t>(va >> 32) & 0xFFFFu, nrec, static_cast<uint32_t>(kRsrcWord3)};
#pragma unroll
        for (int j = 0; j < G::NLW; ++j) {
            const int b = w + j * kWaves;                 // scalar: which 1 KiB block of the tile
            if (b < G::NB) {
                const int so = b * G::RPW * rs32;
                if constexpr (FUSED) {
                    if (straddle) {
                        // At most once per work item, and only when `off` is not a multiple of the tile.  Lanes whose
                        // row lies below `off` load from the cache, the others from the new rows (a resource whose
                        // row 0 is position `tok`); a lane that is switched off writes nothing to LDS (checked on
                        // the chip), so the two loads fill disjoint parts of the block.
                        const uint64_t nka = reinterpret_cast<uint64_t>(kn) + static_cast<int64_t>(tok - off) * ns32;
                        const uint64_t nva = reinterpret_cast<uint64_t>(vn) + static_cast<int64_t>(tok - off) * ns32;
                        const uint32_t nnrec = static_cast<uint32_t>((rows - 1) * ns32 + G::RB);
                        const u32x4 nkrs = {static_cast<uint32_t>(nka), static_cast<uint32_t>(nka >> 32) & 0xFFFFu, nnrec, static_cast<uint32_t>(kRsrcWord3)};
                        const u32x4 nvrs = {static_cast<uint32_t>(nva), static_cast<uint32_t>(nva >> 32) & 0xFFFFu, nnrec, static_cast<uint32_t>(kRsrcWord3)};
                        if (tok + b * G::RPW + dma_row < off) {
                            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                                         :: "s"(kb + b * 1024), "v"(dma_voff_k[((j * kWaves) % PB) / STEP]), "s"(krs), "s"(so) : "memory", "m0");
                            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                                         :: "s"(kb + G::KV + b * 1024), "v"(dma_voff_v), "s"(vrs), "s"(so) : "memory", "m0");
                        } else {
                            const int nso = b * G::RPW * ns32;
                            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                                         :: "s"(kb + b * 1024), "v"(dma_voff_k[((j * kWaves) % PB) / STEP] - dma_row_excess), "s"(nkrs), "s"(nso) : "memory", "m0");
                            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                                         :: "s"(kb + G::KV + b * 1024), "v"(dma_voff_v - dma_row_excess), "s"(nvrs), "s"(nso) : "memory", "m0");
                        }
                        continue;
                    }
                }
                asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                             :: "s"(kb + b * 1024), "v"(dma_voff_k[((j * kWaves) % PB) / STEP]), "s"(krs), "s"(so) : "memory", "m0");
                asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                             :: "s"(kb + G::KV + b * 1024), "v"(dma_voff_v), "s"(vrs), "s"(so) : "memory", "m0");
            }
        }
    };

    const float scale_log2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.f;
    f32x16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

    const int wave_last_key = min(row_lo + WR - 1, q_len - 1) + off;  // last key any row of the wave sees
    // Per-lane LDS read offsets under the chunk permutations.  K fragment (k-step ks): lane reads row l%32
    // (+32 for the second token half), logical chunk 2*ks + l/32.  V fragment (channel block db): lane
    // reads 8 bytes of row vrow (+8, +16, +32) inside the logical 64-byte group db.  In both cases the
    // row's permutation value depends on the lane only.
    int koff[D / 16], voff[D / 32];
    {
        const int sk = G::swz_k(l & 31);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) koff[ks] = (l & 31) * G::RB + (((2 * ks + (l >> 5)) ^ sk) << 4);
        const int vrow = (l >> 5) * 4 + ((l & 15) >> 2);
        const int sv = G::swz_v(vrow) >> 2;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) voff[db] = vrow * G::RB + ((db ^ sv) << 6) + ((l >> 4) & 1) * 32 + (l & 3) * 8;
    }

    // One KV tile in two parts, S^T = K Q^T first, then online softmax and O^T += V^T P^T.
    f32x16 s[2];
    auto wave_active = [&](int t) { return t * kBN <= wave_last_key && row_lo < q_len; };
    auto tile_scores = [&](int t) {
        const char* kb = lds + (t & (G::STAGES - 1)) * G::BUF;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[tb][i] = 0.f;
        // operands are fetched several multiplies ahead so the matrix pipe is not paced by LDS latency;
        // the wave runs at raised priority while it feeds the matrix pipe
        __builtin_amdgcn_s_setprio(1);
        constexpr int NF = D / 16 * 2;       // K fragments of the tile
        bf16x8 ka[NF];
#pragma unroll
        for (int f = 0; f < NF; ++f)
            ka[f] = *reinterpret_cast<const bf16x8*>(kb + (f & 1) * 32 * G::RB + koff[f >> 1]);
#pragma unroll
        for (int f = 0; f < NF; ++f)
            s[f & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[f], qb[f >> 1], s[f & 1], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
        for (int f = 0; f < NF - kAhead; ++f) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
        __builtin_amdgcn_s_setprio(0);
    };
    auto tile_softmax_pv = [&](int t) {
        const char* vb = lds + (t & (G::STAGES - 1)) * G::BUF + G::KV;
        const int t0 = t * kBN;
        bf16x8 pb[4];
        // lane owns query row my_row; s[tb][i] is token t0 + tb*32 + (i/4)*8 + (l/32)*4 + i%4
        if (t0 + kBN - 1 > row_lo + off) {             // tile crosses the diagonal for some row of the wave
            const int limit = my_row + off;            // last visible key of this lane's row
            const int tl = t0 + (l >> 5) * 4;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (tl + tb * 32 + (i >> 2) * 8 + (i & 3) > limit) s[tb][i] = -INFINITY;
        }
        float mx = s[0][0];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[tb][i]);
        // the row's other half lives in lane l ^ 32: v_permlane32_swap exchanges the wave halves of two
        // registers in the vector unit (a cross-lane shuffle would go through LDS and its latency sits on
        // the critical path of the softmax); scale > 0: max commutes with scaling
        {
            const unsigned bits = __builtin_bit_cast(unsigned, mx);
            const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);   // {lo,lo}, {hi,hi}
            mx = fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1])) * scale_log2;
        }
        // Query rows past q_len hold a copy of the last row's Q, and key 0 is visible to every row, so
        // the first tile always raises m from -inf to a finite value for all lanes.
        if (__builtin_amdgcn_ballot_w64(mx > m + kLazy) != 0) {
            const float m_new = fmaxf(m, mx);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
        }
        const float neg_m = -m;
        float lpart[2] = {0.f, 0.f};
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[tb][i], scale_log2, neg_m));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[tb][i + 1], scale_log2, neg_m));
                // row sum in fp32 with plain adds (the bf16 dot-product instruction shares hardware with the
                // matrix pipe and stalls it); two partial sums keep the chains short
                lpart[tb] += p0 + p1;
                pb[tb * 2 + (i >> 3)][i & 7] = static_cast<__bf16>(p0);
                pb[tb * 2 + (i >> 3)][(i & 7) + 1] = static_cast<__bf16>(p1);
            }
        lsum += lpart[0] + lpart[1];

        // O^T += V^T P^T.  A operand: lane (d = db*32 + l%32, h = l/32), 8 tokens per k-step (kk = tb*2 + s').
        __builtin_amdgcn_s_setprio(1);
        constexpr int NV = 4 * (D / 32);
        s16x4 vlo[NV], vhi[NV];
#pragma unroll
        for (int f = 0; f < NV; ++f) {
            const int kk = f / (D / 32), db = f % (D / 32);
            const char* p0 = vb + ((kk >> 1) * 32 + (kk & 1) * 16) * G::RB + voff[db];
            vlo[f] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
            vhi[f] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * G::RB));
        }
#pragma unroll
        for (int f = 0; f < NV; ++f) {
            const int kk = f / (D / 32), db = f % (D / 32);
            const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(vlo[f], vhi[f], 0, 1, 2, 3, 4, 5, 6, 7));
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kk], o[db], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
        for (int f = 0; f < NV - kAhead; ++f) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kAhead, 0);
        __builtin_amdgcn_s_setprio(0);
    };

    // Four-stage LDS ring, tile x in stage x % 4, walked two tiles per iteration: one workgroup barrier per
    // 128 tokens.  Tiles t+2 and t+3 go into the stages of tiles t-2 and t-1, which every wave finished
    // reading before the last barrier; a tile index past the end is out of range for every lane and only
    // writes zeros.
    issue_loads(0);
    issue_loads(1);
    // everything requested so far - Q and the first two tiles - has landed before the loop starts
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
    __syncthreads();

    for (int t = 0; t < ntiles; t += 2) {
        issue_loads(t + 2);
        issue_loads(t + 3);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (wave_active(t + u)) {     // false for t + u >= ntiles as well
                tile_scores(t + u);
                tile_softmax_pv(t + u);
            }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // this wave's parts of the two new tiles are in LDS
        __syncthreads();
    }

    lsum += __shfl_xor(lsum, 32);
    if (my_row < q_len) {
        const float inv = 1.f / lsum;
        char* orow = static_cast<char*>(a.o) + ((static_cast<int64_t>(q_begin) + my_row) * a.Hq + head) * G::RB;
        // A lane holds 4 consecutive channels of its row per group of 8, the lane 32 further on the other 4.  The two
        // trade every second group (one cross-half swap per register), so that each stores 8 consecutive channels:
        // half as many store instructions, twice as wide.
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                bf16x4 ve, vo;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ve[e] = static_cast<__bf16>(o[db][(2 * pr) * 4 + e] * inv);
                    vo[e] = static_cast<__bf16>(o[db][(2 * pr + 1) * 4 + e] * inv);
                }
                const u32x2 e2 = __builtin_bit_cast(u32x2, ve), o2 = __builtin_bit_cast(u32x2, vo);
                // swap(E, O): the lower half keeps its own E and receives the upper half's E; the upper half
                // receives the lower half's O and keeps its own O
                const auto s0 = __builtin_amdgcn_permlane32_swap(e2[0], o2[0], false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(e2[1], o2[1], false, false);
                const u32x4 out = {s0[0], s1[0], s0[1], s1[1]};
                const int d = db * 32 + (2 * pr + (l >> 5)) * 8;
                *reinterpret_cast<u32x4*>(orow + d * 2) = out;
            }
    }
    __syncthreads();   // every wave is done with the LDS ring and with sh_item
  }
}

}  // namespace

bool launch_prefill(const PrefillArgs& a_in, hipStream_t stream, LaunchEvents ev) {
    const int group = a_in.Hq / a_in.H;
    const unsigned all_slots = static_cast<unsigned>(8 * a_in.items_per_xcd * group);
    if (all_slots == 0) return true;
    const PrefillArgs& a = a_in;
    // Persistent workgroups: as many as the chip keeps resident (asked of the runtime once per kernel
    // variant), a multiple of 8 so that every XCD gets the same number; each drains the queues by itself.
    static int resident_per_cu[8] = {};  // per kernel variant; 0 = not asked yet
    auto launch = [&](auto kernel, int lds, int variant) -> bool {
        const int threads = a.waves * 64;
        if (resident_per_cu[variant] == 0) {
            // dynamic LDS above 64 KiB has to be allowed once per kernel
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds), "hipFuncSetAttribute")) return false;
            int per_cu = 0;
            if (!hip_ok(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, static_cast<size_t>(lds)), "hipOccupancyMaxActiveBlocksPerMultiprocessor")) return false;
            resident_per_cu[variant] = per_cu > 0 ? per_cu : 1;
        }
        const unsigned resident = static_cast<unsigned>(resident_per_cu[variant] * a.num_cus) / 8u * 8u;
        const dim3 grid(all_slots < resident ? all_slots : (resident ? resident : 8u));
        hipExtLaunchKernelGGL(kernel, grid, dim3(static_cast<unsigned>(threads)), static_cast<size_t>(lds), stream, ev.start, ev.stop, 0, a);
        return true;
    };
    bool ok;
    if (a.k_new) {
        if (a.waves == 12) ok = a.D == 128 ? launch(prefill_kernel<128, 12, true>, PGeo<128, 12>::LDS, 6) : launch(prefill_kernel<64, 12, true>, PGeo<64, 12>::LDS, 7);
        else ok = a.D == 128 ? launch(prefill_kernel<128, 8, true>, PGeo<128, 8>::LDS, 4) : launch(prefill_kernel<64, 8, true>, PGeo<64, 8>::LDS, 5);
    } else if (a.waves == 12) ok = a.D == 128 ? launch(prefill_kernel<128, 12, false>, PGeo<128, 12>::LDS, 2) : launch(prefill_kernel<64, 12, false>, PGeo<64, 12>::LDS, 3);
    else ok = a.D == 128 ? launch(prefill_kernel<128, 8, false>, PGeo<128, 8>::LDS, 0) : launch(prefill_kernel<64, 8, false>, PGeo<64, 8>::LDS, 1);
    if (!ok) return false;
    return hip_ok(hipGetLastError(), "prefill launch");
}

}  // namespace vattn
