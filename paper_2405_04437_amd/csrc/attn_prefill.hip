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

#include "vattn_internal.h"

namespace vattn {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kBM = 128;   // query rows per workgroup
constexpr int kBN = 64;    // KV tokens per tile
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

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
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int w = tid >> 6;
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
    const int q0 = it.q_tile * kBM;
    const int q_last = min(q0 + kBM, q_len) - 1;
    const int n_kv = q_last + off + 1;         // keys any row of this tile can see
    const int ntiles = (n_kv + kBN - 1) / kBN;

    const int64_t row_stride = static_cast<int64_t>(a.H) * G::RB;
    const int64_t sub = static_cast<int64_t>(a.reqids[req]) * a.S + static_cast<int64_t>(it.kvh) * G::RB;
    const char* kp = a.k_base + sub;
    const char* vp = a.v_base + sub;

    // Q^T as B operand: lane (n = l%32, h = l/32) holds Q[row n][ks*16 + h*8 .. +8]
    const int my_row = q0 + w * 32 + (l & 31);
    bf16x8 qb[D / 16];
    {
        const int qr = min(my_row, q_len - 1);
        const char* qrow = static_cast<const char*>(a.q) + ((static_cast<int64_t>(q_begin) + qr) * a.Hq + head) * G::RB;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            qb[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + ks * 32 + (l >> 5) * 16));
    }

    const int ld_row = tid / G::LPR;
    const int ld_col = (tid % G::LPR) * 16;
    u32x4 kreg[G::NL], vreg[G::NL];
    auto issue_loads = [&](int t) {
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int tok = min(t * kBN + i * G::RPI + ld_row, kv_len - 1);  // never beyond the mapped context
            const int64_t o = static_cast<int64_t>(tok) * row_stride + ld_col;
            kreg[i] = *reinterpret_cast<const u32x4*>(kp + o);
            vreg[i] = *reinterpret_cast<const u32x4*>(vp + o);
        }
    };
    auto store_tile = [&](int buf) {
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
    float m = -INFINITY, lsum = 0.f;
    f32x16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

    const int row_lo = q0 + w * 32;               // first query row of this wave
    const int wave_last_key = min(row_lo + 31, q_len - 1) + off;  // last key any row of the wave sees

    issue_loads(0);
    store_tile(0);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const bool more = t + 1 < ntiles;
        if (more) issue_loads(t + 1);
        const char* kb = lds + (t & 1) * G::BUF;
        const char* vb = kb + kBN * G::KSTR;
        const int t0 = t * kBN;
        if (t0 <= wave_last_key && row_lo < q_len) {
            f32x16 s[2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[tb][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const bf16x8 ka = *reinterpret_cast<const bf16x8*>(kb + (tb * 32 + (l & 31)) * G::KSTR + ks * 32 + (l >> 5) * 16);
                    s[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[ks], s[tb], 0, 0, 0);
                }
            // lane owns query row my_row; s[tb][i] is token t0 + tb*32 + (i/4)*8 + (l/32)*4 + i%4
            const bool need_mask = t0 + kBN - 1 > row_lo + off;
            float mx = -INFINITY;
            if (need_mask) {
                const int limit = my_row + off;  // last visible key of this lane's row
                const int tl = t0 + (l >> 5) * 4;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int tok = tl + tb * 32 + (i >> 2) * 8 + (i & 3);
                        float x = s[tb][i] * scale_log2;
                        if (tok > limit) x = -INFINITY;
                        s[tb][i] = x;
                        mx = fmaxf(mx, x);
                    }
            } else {
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float x = s[tb][i] * scale_log2;
                        s[tb][i] = x;
                        mx = fmaxf(mx, x);
                    }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // Rows past q_len are clamped copies of the last row, and key 0 is visible to every row,
            // so after the first tile m is finite for all lanes.
            const float m_new = fmaxf(m, mx);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            float psum = 0.f;
            bf16x8 pb[4];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = __builtin_amdgcn_exp2f(s[tb][i] - m_new);
                    psum += p;
                    pb[tb * 2 + (i >> 3)][i & 7] = static_cast<__bf16>(p);
                }
            lsum = lsum * alpha + psum;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= alpha;

            // O^T += V^T P^T.  A operand: lane (d = db*32 + l%32, h = l/32), 8 tokens per k-step.
            const int vrow = (l >> 5) * 4 + ((l & 15) >> 2);
            const int vcol = ((l >> 4) & 1) * 32 + (l & 3) * 8;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {          // kk = tb*2 + s'
                const int trow = (kk >> 1) * 32 + (kk & 1) * 16 + vrow;
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const char* p0 = vb + trow * G::VSTR + db * 64 + vcol;
                    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
                    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * G::VSTR));
                    const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kk], o[db], 0, 0, 0);
                }
            }
        }
        if (more) store_tile((t + 1) & 1);
        __syncthreads();
    }

    lsum += __shfl_xor(lsum, 32);
    if (my_row < q_len) {
        const float inv = 1.f / lsum;
        char* orow = static_cast<char*>(a.o) + ((static_cast<int64_t>(q_begin) + my_row) * a.Hq + head) * G::RB;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[db][q4 * 4 + e] * inv);
                const int d = db * 32 + q4 * 8 + (l >> 5) * 4;
                *reinterpret_cast<u32x2*>(orow + d * 2) = __builtin_bit_cast(u32x2, v);
            }
    }
}

}  // namespace

int prefill_tile_rows(int, int, int) { return kBM; }
int prefill_heads_per_item(int Hq, int H, int) { return Hq / H; }

bool launch_prefill(const PrefillArgs& a, hipStream_t stream) {
    const int group = a.Hq / a.H;
    dim3 grid(static_cast<unsigned>(8 * a.items_per_xcd * group));
    if (grid.x == 0) return true;
    if (a.D == 128) {
        static bool attr_set = false;
        if (!attr_set) {
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kernel<128>), hipFuncAttributeMaxDynamicSharedMemorySize, PGeo<128>::LDS), "hipFuncSetAttribute")) return false;
            attr_set = true;
        }
        hipLaunchKernelGGL(prefill_kernel<128>, grid, dim3(kThreads), PGeo<128>::LDS, stream, a);
    } else {
        static bool attr_set = false;
        if (!attr_set) {
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kernel<64>), hipFuncAttributeMaxDynamicSharedMemorySize, PGeo<64>::LDS), "hipFuncSetAttribute")) return false;
            attr_set = true;
        }
        hipLaunchKernelGGL(prefill_kernel<64>, grid, dim3(kThreads), PGeo<64>::LDS, stream, a);
    }
    return hip_ok(hipGetLastError(), "prefill launch");
}

}  // namespace vattn
