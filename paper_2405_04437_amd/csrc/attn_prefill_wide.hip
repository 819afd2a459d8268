// Causal prefill attention, wide variant: 256 query rows per workgroup, 64 per wave.
//
// Same computation as attn_prefill.hip (Eq. 2 of the paper per request, causal, GQA, K/V read in place
// from the request's virtually contiguous sub-tensor), arranged for long prompts:
//
//  * Each wave owns two 32-row query blocks, so every K and V fragment read from LDS feeds two
//    v_mfma_f32_32x32x16_bf16 instead of one.  With one block per wave the LDS has to deliver about
//    128 B/clk/CU at the matrix peak, more than half of the ~215 B/clk measured for it; with two it is
//    half of that, and a 256-row workgroup also halves the K/V bytes each CU pulls through L2.
//  * The price is registers (two output accumulators, two Q fragment sets): one wave per SIMD.  With no
//    second wave to hide behind, matrix and vector work are interleaved inside the wave: the KV sequence
//    is walked in half-steps of 32 tokens, and while the score multiplies of half-step h+1 are in the
//    matrix pipe the vector unit does the softmax of half-step h (software pipeline, scores ping-pong
//    between two register sets).  The pipelined loop covers the half-steps that lie entirely below the
//    workgroup's diagonal; the few diagonal half-steps run through a plain masked path.
//  * K/V tiles of 64 tokens sit in a three-stage LDS ring: tile T+2 is requested from global memory at
//    the start of tile T and written to LDS at its end, into the stage tile T-1 was read from (that
//    iteration ended with a barrier).  During tile T the waves read tile T and, for the scores that run
//    one half-step ahead, the first half of tile T+1.  One workgroup barrier per tile.
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

constexpr int kTile = 64;      // KV tokens per LDS tile
constexpr int kHalf = 32;      // KV tokens per half-step
constexpr int kThreads = 256;
constexpr int kBM = 256;       // query rows per workgroup
constexpr int kStages = 3;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.0f;  // rescale only when a row maximum grows by more than 2^8 (see attn_prefill.hip)
constexpr int kRsrcWord3 = 0x00020000;  // gfx9-family raw buffer resource, 32-bit data format

template <int D> struct WGeo {
    static constexpr int RB = D * 2;
    static constexpr int KSTR = RB + 16;
    static constexpr int VSTR = RB + 64;
    static constexpr int LPR = RB / 16;
    static constexpr int RPI = kThreads / LPR;
    static constexpr int NL = kTile / RPI;
    static constexpr int STAGE = kTile * (KSTR + VSTR);
    static constexpr int LDS = kStages * STAGE;
};

template <int D>
__global__ __launch_bounds__(kThreads, 1) void prefill_wide_kernel(PrefillArgs a) {
    using G = WGeo<D>;
    constexpr int NK = D / 16;   // K fragments (k-steps over the head dimension) per half-step
    constexpr int NDB = D / 32;  // 32-channel output blocks
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63;
    const int group = a.Hq / a.H;

    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const PrefillItem it = a.items[static_cast<int64_t>(xcd) * a.items_per_xcd + slot / group];
    if (it.req < 0) return;
    const int head = it.kvh * group + slot % group;
    const int req = it.req;
    const int q_begin = a.cu_q[req];
    const int q_len = a.cu_q[req + 1] - q_begin;
    const int kv_len = a.kv_lens[req];
    const int off = kv_len - q_len;
    const int q0 = it.q_tile * kBM;
    const int q_last = min(q0 + kBM, q_len) - 1;
    const int n_kv = q_last + off + 1;
    const int ntiles = (n_kv + kTile - 1) / kTile;
    // half-steps whose 32 tokens are visible to every row of the workgroup (no mask, no skipping)
    const int h_full = (q0 + off + 1) / kHalf;
    // tiles both of whose half-steps can be pipelined (the step after each is still unmasked)
    const int tiles_piped = h_full >= 2 ? (h_full - 1) / 2 : 0;

    const int rs32 = a.row_stride;             // bytes between consecutive tokens of this layer
    const int64_t sub = static_cast<int64_t>(a.reqids[req]) * a.S + static_cast<int64_t>(it.kvh) * G::RB;
    const char* kp = a.k_base + sub;
    const char* vp = a.v_base + sub;

    const int row_lo = q0 + w * 64;
    int my_row[2];
    bf16x8 qb[2][NK];
#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        my_row[qa] = row_lo + qa * 32 + (l & 31);
        const int qr = min(my_row[qa], q_len - 1);
        const char* qrow = static_cast<const char*>(a.q) + ((static_cast<int64_t>(q_begin) + qr) * a.Hq + head) * G::RB;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks)
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
    u32x4 kreg[G::NL], vreg[G::NL];
    auto issue_loads = [&](int T) {
        const int tok = T * kTile;
        const int64_t boff = static_cast<int64_t>(tok) * rs32;
        const int rows = min(kv_len - tok, kTile);   // <= 0 past the end: everything out of range
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
    auto store_tile = [&](int stage) {
        char* kb = lds + stage * G::STAGE;
        char* vb = kb + kTile * G::KSTR;
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int row = i * G::RPI + ld_row;
            *reinterpret_cast<u32x4*>(kb + row * G::KSTR + ld_col) = kreg[i];
            *reinterpret_cast<u32x4*>(vb + row * G::VSTR + ld_col) = vreg[i];
        }
    };

    const float scale_log2 = a.scale * kLog2e;
    float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.f, 0.f};
    f32x16 o[2][NDB];
#pragma unroll
    for (int qa = 0; qa < 2; ++qa)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[qa][db][i] = 0.f;

    const int wave_last_key = min(row_lo + 63, q_len - 1) + off;
    const int kfrag_off = (l & 31) * G::KSTR + (l >> 5) * 16;          // lane part of a K fragment address
    const int vfrag_off = ((l >> 5) * 4 + ((l & 15) >> 2)) * G::VSTR + ((l >> 4) & 1) * 32 + (l & 3) * 8;
    bf16x2 ones;
    ones[0] = static_cast<__bf16>(1.0f);
    ones[1] = static_cast<__bf16>(1.0f);

    // ---- building blocks (h = half-step index; its tokens are rows (h&1)*32.. of tile h/2) --------------
    // The per-lane base of a half-step is passed through an empty asm so that the compiler keeps it as
    // ONE register and folds every fragment's constant displacement into the ds_read offset field
    // (otherwise it hoists one address register per fragment out of the loop and re-adds the stage
    // offset to each of them every half-step).
    auto lds_base = [&](int byte_off) {
        uint32_t a32 = static_cast<uint32_t>(byte_off);
        asm volatile("" : "+v"(a32));
        return reinterpret_cast<const char*>(lds) + a32;
    };
    auto k_half = [&](int h) { return lds_base(((h >> 1) % kStages) * G::STAGE + (h & 1) * kHalf * G::KSTR + kfrag_off); };
    auto v_half = [&](int h) { return lds_base(((h >> 1) % kStages) * G::STAGE + kTile * G::KSTR + (h & 1) * kHalf * G::VSTR + vfrag_off); };

    auto zero_scores = [&](f32x16 (&s)[2]) {
#pragma unroll
        for (int qa = 0; qa < 2; ++qa)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[qa][i] = 0.f;
    };
    // row maximum of one 32-token score block, scaled to the log2 domain
    auto row_max = [&](const f32x16& s) {
        float mx = s[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
        const unsigned bits = __builtin_bit_cast(unsigned, mx);
        const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);   // wave halves exchanged in the vector unit
        return fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1])) * scale_log2;
    };
    auto rescale = [&](int qa, float mx) {
        const float m_new = fmaxf(m[qa], mx);
        const float alpha = __builtin_amdgcn_exp2f(m[qa] - m_new);
        m[qa] = m_new;
        lsum[qa] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[qa][db][i] *= alpha;
    };
    // probabilities of one block: p = 2^(s*c - m), rounded to bf16; the row sum uses the rounded values
    auto probs = [&](int qa, const f32x16& s, bf16x8 (&pb)[2]) {
        const float neg_m = -m[qa];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            bf16x2 pp;
            pp[0] = static_cast<__bf16>(__builtin_amdgcn_exp2f(__builtin_fmaf(s[i], scale_log2, neg_m)));
            pp[1] = static_cast<__bf16>(__builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 1], scale_log2, neg_m)));
            lsum[qa] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, lsum[qa], false);
            pb[i >> 3][i & 7] = pp[0];
            pb[i >> 3][(i & 7) + 1] = pp[1];
        }
    };
    // O^T += V^T P^T for one half-step: 2 k-steps of 16 tokens x NDB channel blocks x 2 query blocks
    auto pv_half = [&](int h, const bf16x8 (&pb)[2][2]) {
        const char* vb = v_half(h);
        s16x4 vlo[2 * NDB], vhi[2 * NDB];
#pragma unroll
        for (int f = 0; f < 2 * NDB; ++f) {
            const char* p0 = vb + (f / NDB) * 16 * G::VSTR + (f % NDB) * 64;
            vlo[f] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
            vhi[f] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * G::VSTR));
        }
#pragma unroll
        for (int f = 0; f < 2 * NDB; ++f) {
            const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(vlo[f], vhi[f], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int qa = 0; qa < 2; ++qa)
                o[qa][f % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[qa][f / NDB], o[qa][f % NDB], 0, 0, 0);
        }
        // first four fragments' reads up front, then two multiplies per fragment with the next reads behind them
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
        for (int f = 0; f < 2 * NDB - 4; ++f) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    };
    // plain score computation of half-step h (used by the prologue and the masked path)
    auto scores_half = [&](int h, f32x16 (&s)[2]) {
        const char* kb = k_half(h);
        zero_scores(s);
        bf16x8 ka[NK];
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) ka[ks] = *reinterpret_cast<const bf16x8*>(kb + ks * 32);
#pragma unroll
        for (int ks = 0; ks < NK; ++ks)
#pragma unroll
            for (int qa = 0; qa < 2; ++qa) s[qa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qb[qa][ks], s[qa], 0, 0, 0);
    };
    // Pipelined half-step: softmax of s_cur (half-step h) on the vector unit while the matrix pipe computes
    // s_nxt = scores of half-step h+1; then the second contraction of half-step h.
    auto fused_step = [&](int h, f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2]) {
        const char* kb = k_half(h + 1);
        bf16x8 ka[NK];
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) ka[ks] = *reinterpret_cast<const bf16x8*>(kb + ks * 32);
        zero_scores(s_nxt);
        // part 1: first two k-steps of the next scores || row maxima of the current ones
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int qa = 0; qa < 2; ++qa) s_nxt[qa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qb[qa][ks], s_nxt[qa], 0, 0, 0);
        const float mx0 = row_max(s_cur[0]);
        const float mx1 = row_max(s_cur[1]);
        if (__builtin_amdgcn_ballot_w64(mx0 > m[0] + kLazy || mx1 > m[1] + kLazy) != 0) {  // rare after the first steps
            rescale(0, mx0);
            rescale(1, mx1);
        }
        // part 2: remaining k-steps || exponentials, bf16 packing and row sums
#pragma unroll
        for (int ks = 2; ks < NK; ++ks)
#pragma unroll
            for (int qa = 0; qa < 2; ++qa) s_nxt[qa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qb[qa][ks], s_nxt[qa], 0, 0, 0);
        bf16x8 pb[2][2];
        probs(0, s_cur[0], pb[0]);
        probs(1, s_cur[1], pb[1]);
#pragma unroll
        for (int f = 0; f < 2 * (NK - 2); ++f) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 96 / (2 * (NK - 2)), 0);
            __builtin_amdgcn_sched_group_barrier(0x400, (32 + 2 * (NK - 2) - 1) / (2 * (NK - 2)), 0);
        }
        pv_half(h, pb);
    };
    // Masked, unpipelined half-step (diagonal region): skipped by waves whose rows see none of its tokens.
    auto plain_step = [&](int h, f32x16 (&s)[2], bool have_scores) {
        const int t0 = h * kHalf;
        if (!(t0 <= wave_last_key && row_lo < q_len)) return;
        if (!have_scores) scores_half(h, s);
        bf16x8 pb[2][2];
#pragma unroll
        for (int qa = 0; qa < 2; ++qa) {
            if (t0 + kHalf - 1 > row_lo + qa * 32 + off) {   // crosses the diagonal for some row of this block
                const int limit = my_row[qa] + off;
                const int tl = t0 + (l >> 5) * 4;
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (tl + (i >> 2) * 8 + (i & 3) > limit) s[qa][i] = -INFINITY;
            }
            const float mx = row_max(s[qa]);
            // key 0 is visible to every row, so the very first half-step makes m finite for all lanes
            if (__builtin_amdgcn_ballot_w64(mx > m[qa] + kLazy) != 0) rescale(qa, mx);
            probs(qa, s[qa], pb[qa]);
        }
        pv_half(h, pb);
    };

    // ---- prologue: tiles 0 and 1 into the ring ----------------------------------------------------------
    issue_loads(0);
    store_tile(0);
    issue_loads(1);
    store_tile(1);
    __syncthreads();
    // All loads issued so far (Q among them) have landed: no wait for Q is left inside the loops.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
    // Park the Q fragments in accumulation registers.  The matrix instructions read their B operand
    // from there directly, and the 64 architectural registers they would occupy are what the softmax
    // needs; left to itself the allocator spills them there anyway but copies them back before every
    // multiply.
#pragma unroll
    for (int qa = 0; qa < 2; ++qa)
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            u32x4 raw = __builtin_bit_cast(u32x4, qb[qa][ks]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t acc;
                asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(acc) : "v"(raw[e]));
                raw[e] = acc;
            }
            qb[qa][ks] = __builtin_bit_cast(bf16x8, raw);
        }

    f32x16 sA[2], sB[2];
    int T = 0;
    bool have = false;   // sA already holds the scores of half-step 2*T
    if (tiles_piped > 0) {
        scores_half(0, sA);
        for (; T < tiles_piped; ++T) {
            issue_loads(T + 2);
            fused_step(2 * T, sA, sB);
            fused_step(2 * T + 1, sB, sA);
            store_tile((T + 2) % kStages);
            __syncthreads();
        }
        have = true;
    }
    // diagonal region; the first of its half-steps may already have its scores (left by the pipeline)
    for (; T < ntiles; ++T) {
        issue_loads(T + 2);
        plain_step(2 * T, sA, have);
        have = false;
        plain_step(2 * T + 1, sA, false);
        store_tile((T + 2) % kStages);
        __syncthreads();
    }

#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        lsum[qa] += __shfl_xor(lsum[qa], 32);
        if (my_row[qa] < q_len) {
            const float inv = 1.f / lsum[qa];
            char* orow = static_cast<char*>(a.o) + ((static_cast<int64_t>(q_begin) + my_row[qa]) * a.Hq + head) * G::RB;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
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

bool launch_prefill_wide(const PrefillArgs& a, hipStream_t stream, LaunchEvents ev) {
    const int group = a.Hq / a.H;
    dim3 grid(static_cast<unsigned>(8 * a.items_per_xcd * group));
    if (grid.x == 0) return true;
    static bool allowed[2] = {false, false};
    auto launch = [&](auto kernel, int lds, int variant) -> bool {
        if (!allowed[variant]) {  // dynamic LDS above 64 KiB has to be allowed once per kernel
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds), "hipFuncSetAttribute")) return false;
            allowed[variant] = true;
        }
        hipExtLaunchKernelGGL(kernel, grid, dim3(kThreads), static_cast<size_t>(lds), stream, ev.start, ev.stop, 0, a);
        return true;
    };
    if (!(a.D == 128 ? launch(prefill_wide_kernel<128>, WGeo<128>::LDS, 0) : launch(prefill_wide_kernel<64>, WGeo<64>::LDS, 1))) return false;
    return hip_ok(hipGetLastError(), "prefill (wide) launch");
}

}  // namespace vattn
