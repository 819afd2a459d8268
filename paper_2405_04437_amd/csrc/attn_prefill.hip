// Causal prefill attention over virtually contiguous KV.
//
// Computes Eq. 2 of the paper per request, o_i = softmax(q_i K^T * scale) V over the keys visible to
// query row i (keys 0 .. kv_len - q_len + i), with K and V read in place from the request's
// sub-tensor at base + reqId*S (Sec. 5.2.3): no block table, one pointer and one stride.
//
// gfx950 mapping
//  * One workgroup (4 waves) owns 128 query rows of one query head; each wave owns 32 rows.  KV is
//    walked in tiles of 64 tokens, staged in LDS (double buffered; global loads for tile t+1 are in
//    flight in registers while tile t is being multiplied).
//  * Both contractions use v_mfma_f32_32x32x16_bf16.  Scores are produced transposed,
//    S^T = K Q^T (tokens x rows): a lane then owns ONE query row, so the running max / sum are
//    per-lane scalars (one cross-lane exchange per tile), and exp(S^T) is already laid out as the B
//    operand of O^T = V^T P^T.  V^T comes out of LDS through ds_read_b64_tr_b16.
//  * The launch is XCD-aware: workgroup ids are dealt round-robin to the 8 XCDs by the hardware, so
//    the host builds one work queue per XCD and gives each XCD whole (request, KV head) streams; the
//    query heads of a group and neighbouring query tiles then run on the same XCD at the same time
//    and share the K/V stream through that XCD's L2.
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
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
// The running maximum is only raised when some row's tile maximum exceeds it by more than this many
// binary orders of magnitude: exponentials then stay below 2^kLazy, which fp32 sums and bf16 P hold
// easily, and the O accumulator is rescaled a handful of times per row instead of once per tile.
constexpr float kLazy = 8.0f;
// Fourth dword of a gfx9-family raw buffer resource: 32-bit data format, no swizzle, no stride.
constexpr int kRsrcWord3 = 0x00020000;

template <int D> struct PGeo {
    static constexpr int RB = D * 2;                         // bytes per head row
    static constexpr int KSTR = RB + 16;                     // K row stride in LDS
    static constexpr int VSTR = RB + 64;                     // V row stride in LDS
    static constexpr int LPR = RB / 16;                      // lanes per row for global loads
    static constexpr int RPI = kThreads / LPR;               // rows per load instruction
    static constexpr int NL = kBN / RPI;                     // load instructions per tile per tensor
    static constexpr int BUF = kBN * (KSTR + VSTR);          // one K+V stage
    static constexpr int LDS = 2 * BUF;
};

template <int D>
__global__ __launch_bounds__(kThreads, 2) void prefill_kernel(PrefillArgs a) {
    using G = PGeo<D>;
    constexpr int QB = 1;                      // 32-row query blocks per wave (the wide kernel has two)
    constexpr int BM = 128 * QB;               // query rows per workgroup
    constexpr int WR = 32 * QB;                // query rows per wave
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform per wave: keeps row/tile arithmetic scalar
    const int l = tid & 63;
    const int group = a.Hq / a.H;

    // work item: queue of this XCD, slot bid/8; the heads of a group are adjacent slots
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const PrefillItem it = a.items[static_cast<int64_t>(xcd) * a.items_per_xcd + slot / group];
    if (it.req < 0) return;  // padding entry (uniform for the whole workgroup)
    const int head = it.kvh * group + slot % group;
    const int req = it.req;
    const int q_begin = a.cu_q[req];
    const int q_len = a.cu_q[req + 1] - q_begin;
    const int kv_len = a.kv_lens[req];
    const int off = kv_len - q_len;            // query row i sees keys 0 .. i + off
    const int q0 = it.q_tile * BM;
    const int q_last = min(q0 + BM, q_len) - 1;
    const int n_kv = q_last + off + 1;         // keys any row of this tile can see
    const int ntiles = (n_kv + kBN - 1) / kBN;

    const int rs32 = a.row_stride;             // bytes between consecutive tokens of this layer
    const int64_t sub = static_cast<int64_t>(a.reqids[req]) * a.S + static_cast<int64_t>(it.kvh) * G::RB;
    const char* kp = a.k_base + sub;
    const char* vp = a.v_base + sub;

    // Q^T as B operand: lane (n = l%32, h = l/32) holds Q[row n][ks*16 + h*8 .. +8], per query block
    const int row_lo = q0 + w * WR;               // first query row of this wave
    int my_row[QB];
    bf16x8 qb[QB][D / 16];
#pragma unroll
    for (int qa = 0; qa < QB; ++qa) {
        my_row[qa] = row_lo + qa * 32 + (l & 31);
        const int qr = min(my_row[qa], q_len - 1);
        const char* qrow = static_cast<const char*>(a.q) + ((static_cast<int64_t>(q_begin) + qr) * a.Hq + head) * G::RB;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qb[qa][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + ks * 32 + (l >> 5) * 16));
    }

    const int ld_row = tid / G::LPR;
    const int ld_col = (tid % G::LPR) * 16;
    // Global addressing: each tile of K and V is a raw buffer resource whose 64-bit base is scalar
    // arithmetic (sub-tensors of any size are addressable); the loads add one per-lane offset, the same
    // for the whole kernel, and a scalar offset per instruction.  num_records ends at the last row of
    // the context: rows past it fail the hardware range check, return zeros and touch nothing, so no
    // byte beyond what step() has mapped is read (their scores are masked).
    const int lane_off = ld_row * rs32 + ld_col;
    // One register set stages the next tile: it is requested right after the score multiplies of tile t
    // have been issued and written to the other LDS buffer at the end of the iteration.  The issue is
    // unconditional (a tile index past the end is out of range for every lane and loads zeros without
    // touching memory) and sits at one place in the loop, which lets the compiler keep the loads in
    // flight across the softmax and the second contraction.
    u32x4 kregA[G::NL], vregA[G::NL];
    auto issue_loads = [&](u32x4 (&kreg)[G::NL], u32x4 (&vreg)[G::NL], int t) {
        const int tok = t * kBN;
        const int64_t boff = static_cast<int64_t>(tok) * rs32;
        const int rows = min(kv_len - tok, kBN);   // <= 0 past the end: everything out of range
        const int nrec = rows > 0 ? (rows - 1) * rs32 + G::RB : 0;
        const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kp + boff), 0, nrec, kRsrcWord3);
        const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vp + boff), 0, nrec, kRsrcWord3);
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int so = i * G::RPI * rs32;
            kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(krs, lane_off, so, 0);
            vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(vrs, lane_off, so, 0);
        }
    };
    auto store_tile = [&](const u32x4 (&kreg)[G::NL], const u32x4 (&vreg)[G::NL], int buf) {
        char* kb = lds + buf * G::BUF;
        char* vb = kb + kBN * G::KSTR;
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int row = i * G::RPI + ld_row;
            *reinterpret_cast<u32x4*>(kb + row * G::KSTR + ld_col) = kreg[i];
            *reinterpret_cast<u32x4*>(vb + row * G::VSTR + ld_col) = vreg[i];
        }
    };

    const float scale_log2 = a.scale * kLog2e;
    float m[QB], lsum[QB];
    f32x16 o[QB][D / 32];
#pragma unroll
    for (int qa = 0; qa < QB; ++qa) {
        m[qa] = -INFINITY;
        lsum[qa] = 0.f;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[qa][db][i] = 0.f;
    }

    const int wave_last_key = min(row_lo + WR - 1, q_len - 1) + off;  // last key any row of the wave sees
    const int vrow = (l >> 5) * 4 + ((l & 15) >> 2);
    const int vcol = ((l >> 4) & 1) * 32 + (l & 3) * 8;

    // One KV tile in two parts, S^T = K Q^T first, then online softmax and O^T += V^T P^T; the caller
    // issues the global prefetch between the two (one issue site, whether or not the wave skips a tile
    // that lies entirely above its diagonal).
    f32x16 s[QB][2];
    auto wave_active = [&](int t) { return t * kBN <= wave_last_key && row_lo < q_len; };
    auto tile_scores = [&](int t) {
        const char* kb = lds + (t & 1) * G::BUF;
#pragma unroll
        for (int qa = 0; qa < QB; ++qa)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[qa][tb][i] = 0.f;
        // operands are fetched several multiplies ahead so the matrix pipe is not paced by LDS latency;
        // the wave runs at raised priority while it feeds the matrix pipe
        __builtin_amdgcn_s_setprio(1);
        constexpr int NF = D / 16 * 2;       // K fragments of the tile
        bf16x8 ka[NF];
#pragma unroll
        for (int f = 0; f < NF; ++f)
            ka[f] = *reinterpret_cast<const bf16x8*>(kb + ((f & 1) * 32 + (l & 31)) * G::KSTR + (f >> 1) * 32 + (l >> 5) * 16);
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int qa = 0; qa < QB; ++qa)
                s[qa][f & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[f], qb[qa][f >> 1], s[qa][f & 1], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
        for (int f = 0; f < NF - 6; ++f) {
            __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 6 * QB, 0);
        __builtin_amdgcn_s_setprio(0);
    };
    auto tile_softmax_pv = [&](int t) {
        const char* vb = lds + (t & 1) * G::BUF + kBN * G::KSTR;
        const int t0 = t * kBN;
        bf16x8 pb[QB][4];
#pragma unroll
        for (int qa = 0; qa < QB; ++qa) {
            // lane owns query row my_row[qa]; s[qa][tb][i] is token t0 + tb*32 + (i/4)*8 + (l/32)*4 + i%4
            if (t0 + kBN - 1 > row_lo + qa * 32 + off) {   // tile crosses the diagonal for some row of the block
                const int limit = my_row[qa] + off;        // last visible key of this lane's row
                const int tl = t0 + (l >> 5) * 4;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (tl + tb * 32 + (i >> 2) * 8 + (i & 3) > limit) s[qa][tb][i] = -INFINITY;
            }
            float mx = s[qa][0][0];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[qa][tb][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;   // scale > 0: max commutes with scaling
            // Query rows past q_len hold a copy of the last row's Q, and key 0 is visible to every row, so
            // the first tile always raises m from -inf to a finite value for all lanes.
            if (__builtin_amdgcn_ballot_w64(mx > m[qa] + kLazy) != 0) {
                const float m_new = fmaxf(m[qa], mx);
                const float alpha = __builtin_amdgcn_exp2f(m[qa] - m_new);
                m[qa] = m_new;
                lsum[qa] *= alpha;
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[qa][db][i] *= alpha;
            }
            const float neg_m = -m[qa];
            bf16x2 ones;
            ones[0] = static_cast<__bf16>(1.0f);
            ones[1] = static_cast<__bf16>(1.0f);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    bf16x2 pp;
                    pp[0] = static_cast<__bf16>(__builtin_amdgcn_exp2f(__builtin_fmaf(s[qa][tb][i], scale_log2, neg_m)));
                    pp[1] = static_cast<__bf16>(__builtin_amdgcn_exp2f(__builtin_fmaf(s[qa][tb][i + 1], scale_log2, neg_m)));
                    // the row sum is taken over the rounded probabilities, the same values P V uses
                    lsum[qa] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, lsum[qa], false);
                    pb[qa][tb * 2 + (i >> 3)][i & 7] = pp[0];
                    pb[qa][tb * 2 + (i >> 3)][(i & 7) + 1] = pp[1];
                }
        }

        // O^T += V^T P^T.  A operand: lane (d = db*32 + l%32, h = l/32), 8 tokens per k-step (kk = tb*2 + s').
        __builtin_amdgcn_s_setprio(1);
        constexpr int NV = 4 * (D / 32);
        s16x4 vlo[NV], vhi[NV];
#pragma unroll
        for (int f = 0; f < NV; ++f) {
            const int kk = f / (D / 32), db = f % (D / 32);
            const int trow = (kk >> 1) * 32 + (kk & 1) * 16 + vrow;
            const char* p0 = vb + trow * G::VSTR + db * 64 + vcol;
            vlo[f] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
            vhi[f] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * G::VSTR));
        }
#pragma unroll
        for (int f = 0; f < NV; ++f) {
            const int kk = f / (D / 32), db = f % (D / 32);
            const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(vlo[f], vhi[f], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int qa = 0; qa < QB; ++qa)
                o[qa][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[qa][kk], o[qa][db], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 12, 0);
#pragma unroll
        for (int f = 0; f < NV - 6; ++f) {
            __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 6 * QB, 0);
        __builtin_amdgcn_s_setprio(0);
    };

    issue_loads(kregA, vregA, 0);
    store_tile(kregA, vregA, 0);
    __syncthreads();
    // make sure the Q fragments have landed before the loop, so that no wait for them (which would also
    // wait for younger K/V prefetches) is left inside it
#pragma unroll
    for (int qa = 0; qa < QB; ++qa)
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(qb[qa][ks]));

    for (int t = 0; t < ntiles; ++t) {
        if (wave_active(t)) tile_scores(t);
        issue_loads(kregA, vregA, t + 1);
        if (wave_active(t)) tile_softmax_pv(t);
        store_tile(kregA, vregA, (t + 1) & 1);
        __syncthreads();
    }

#pragma unroll
    for (int qa = 0; qa < QB; ++qa) {
        lsum[qa] += __shfl_xor(lsum[qa], 32);
        if (my_row[qa] < q_len) {
            const float inv = 1.f / lsum[qa];
            char* orow = static_cast<char*>(a.o) + ((static_cast<int64_t>(q_begin) + my_row[qa]) * a.Hq + head) * G::RB;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[qa][db][q4 * 4 + e] * inv);
                    const int d = db * 32 + q4 * 8 + (l >> 5) * 4;
                    *reinterpret_cast<u32x2*>(orow + d * 2) = __builtin_bit_cast(u32x2, v);
                }
        }
    }
}

}  // namespace

bool launch_prefill(const PrefillArgs& a_in, hipStream_t stream, LaunchEvents ev) {
    const int group = a_in.Hq / a_in.H;
    dim3 grid(static_cast<unsigned>(8 * a_in.items_per_xcd * group));
    if (grid.x == 0) return true;
    const PrefillArgs& a = a_in;
    static bool allowed[2] = {false, false};  // per kernel variant
    auto launch = [&](auto kernel, int lds, int variant) -> bool {
        if (!allowed[variant]) {  // dynamic LDS above 64 KiB has to be allowed once per kernel
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds), "hipFuncSetAttribute")) return false;
            allowed[variant] = true;
        }
        hipExtLaunchKernelGGL(kernel, grid, dim3(kThreads), static_cast<size_t>(lds), stream, ev.start, ev.stop, 0, a);
        return true;
    };
    if (!(a.D == 128 ? launch(prefill_kernel<128>, PGeo<128>::LDS, 0) : launch(prefill_kernel<64>, PGeo<64>::LDS, 1))) return false;
    return hip_ok(hipGetLastError(), "prefill launch");
}

}  // namespace vattn
