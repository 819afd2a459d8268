// Decode attention over virtually contiguous KV: split-K kernel + reduce kernel.
//
// What is computed is Eq. 2 of the paper for one query token per request, o = softmax(q K^T * scale) V,
// with K, V read straight from the request's sub-tensor at base + reqId*S (Sec. 5.2.3) - the kernel
// never consults a block table.  The context is cut into fixed-size token chunks; every (chunk,
// KV head) pair is handled by ONE wavefront that keeps a running maximum m, a running sum l and an
// un-normalised output for the query heads of its KV head (the split-K scheme the paper cites as
// FlashDecoding); a second kernel merges the chunk partials.
//
// gfx950 mapping
//  * The path is HBM-bound (8 or 7 flops per KV byte), so the design goal is a deep, fully coalesced
//    load stream: the waves of a workgroup take the KV heads of the SAME token range, so together
//    they read one contiguous byte range of K and one of V.  Every lane loads 16 bytes; a wave has
//    16 such loads in flight (one 32-token tile of K and of V) while it computes the previous tile.
//  * The two contractions run on the matrix cores (v_mfma_f32_16x16x32_bf16).  Scores are computed
//    transposed, S^T = K Q^T (tokens x heads), so that each lane owns one query head: the softmax
//    state is per lane, and the exponentiated scores are already in the register layout the second
//    contraction O^T = V^T P^T wants for its B operand - P never touches LDS.
//  * K and V tiles pass through a wave-private LDS region (no workgroup barrier anywhere): K rows are
//    re-read as 16-byte A operands, V is re-read with the transposing LDS load ds_read_b64_tr_b16,
//    which delivers "8 tokens of one channel" per lane as the A operand of O^T = V^T P^T.
#include <hip/hip_runtime.h>

#include "vattn_internal.h"

namespace vattn {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kTile = 32;          // tokens per inner iteration of a wave
constexpr int kMaxWaves = 8;       // waves (KV heads) per workgroup
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct Geo {
    static constexpr int RB = D * 2;              // bytes of one head row
    static constexpr int LPR = RB / 16;           // lanes per row
    static constexpr int RPI = 64 / LPR;          // rows per load instruction
    static constexpr int NL = kTile / RPI;        // load instructions per tile (per K, per V)
    static constexpr int KSTR = RB + 16;          // LDS row stride of K (bank-conflict-free b128 reads)
    static constexpr int VSTR = RB + 32;          // LDS row stride of V (bank-conflict-free transposed reads)
    static constexpr int WAVE_LDS = kTile * (KSTR + VSTR);
};

__device__ __forceinline__ float xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask)); }

template <int D>
__global__ __launch_bounds__(kMaxWaves * 64) void decode_splitk_kernel(DecodeArgs a, int units, int hb_per_kv) {
    using G = Geo<D>;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int wave = threadIdx.x >> 6;
    const int l = threadIdx.x & 63;
    const int unit = blockIdx.y * (blockDim.x >> 6) + wave;
    if (unit >= units) return;  // no workgroup barrier is ever used, so leaving early is safe
    const int kvh = unit / hb_per_kv;
    const int hb = unit - kvh * hb_per_kv;
    const int group = a.Hq / a.H;

    // which request does this chunk belong to: largest r with cu_chunks[r] <= chunk
    const int chunk = blockIdx.x;
    int lo = 0, hi = a.n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.cu_chunks[mid] <= chunk) lo = mid; else hi = mid;
    }
    const int req = lo;
    const int kv_len = a.kv_lens[req];
    const int tok0 = (chunk - a.cu_chunks[req]) * a.chunk_tokens;
    const int tok1 = min(tok0 + a.chunk_tokens, kv_len);
    const int64_t row_stride = static_cast<int64_t>(a.H) * G::RB;
    const int64_t sub = static_cast<int64_t>(a.reqids[req]) * a.S + static_cast<int64_t>(kvh) * G::RB;
    const char* kp = a.k_base + sub;
    const char* vp = a.v_base + sub;

    char* klds = lds_raw + wave * G::WAVE_LDS;
    char* vlds = klds + kTile * G::KSTR;

    // Query heads of this wave as B operands of S^T = K Q^T: lane (n = l%16, j = l/16) holds
    // Q[head n][kb*32 + j*8 .. +8].
    const int hl = hb * 16 + (l & 15);
    const bool head_ok = hl < group;
    const int head = kvh * group + hl;
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
    u32x4 kreg[G::NL], vreg[G::NL];
    auto issue_loads = [&](int t) {
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            // rows past the end of the context are clamped to the last valid token: never read
            // beyond what step() has mapped; their scores are masked below.
            const int tok = min(tok0 + t * kTile + i * G::RPI + ld_row, kv_len - 1);
            const int64_t off = static_cast<int64_t>(tok) * row_stride + ld_col;
            kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + off));
            vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vp + off));
        }
    };

    const float scale_log2 = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.f;
    f32x4 o[D / 16];
#pragma unroll
    for (int db = 0; db < D / 16; ++db) o[db] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int ntiles = (tok1 - tok0 + kTile - 1) / kTile;
    issue_loads(0);
    for (int t = 0; t < ntiles; ++t) {
#pragma unroll
        for (int i = 0; i < G::NL; ++i) {
            const int row = i * G::RPI + ld_row;
            *reinterpret_cast<u32x4*>(klds + row * G::KSTR + ld_col) = kreg[i];
            *reinterpret_cast<u32x4*>(vlds + row * G::VSTR + ld_col) = vreg[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (t + 1 < ntiles) issue_loads(t + 1);

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
        mx = xor_max(mx, 16);
        mx = xor_max(mx, 32);
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
    }

    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (head_ok) {
        float* po = a.part_o + (static_cast<int64_t>(chunk) * a.Hq + head) * D + (l >> 4) * 4;
#pragma unroll
        for (int db = 0; db < D / 16; ++db) *reinterpret_cast<f32x4*>(po + db * 16) = o[db];
        if ((l >> 4) == 0) {
            float* pml = a.part_ml + (static_cast<int64_t>(chunk) * a.Hq + head) * 2;
            pml[0] = m;
            pml[1] = lsum;
        }
    }
}

// Merge of the chunk partials: with M = max_s m_s,  o = sum_s 2^(m_s-M) o_s / sum_s 2^(m_s-M) l_s.
// One workgroup per (request, query head), one thread per output channel.
template <int D>
__global__ __launch_bounds__(D) void decode_reduce_kernel(DecodeArgs a) {
    const int req = blockIdx.x / a.Hq;
    const int head = blockIdx.x - req * a.Hq;
    const int c0 = a.cu_chunks[req], c1 = a.cu_chunks[req + 1];
    const int d = threadIdx.x;
    float M = -INFINITY;
    for (int c = c0; c < c1; ++c) M = fmaxf(M, a.part_ml[(static_cast<int64_t>(c) * a.Hq + head) * 2]);
    float num = 0.f, den = 0.f;
    for (int c = c0; c < c1; ++c) {
        const int64_t idx = static_cast<int64_t>(c) * a.Hq + head;
        const float w = __builtin_amdgcn_exp2f(a.part_ml[idx * 2] - M);
        den += w * a.part_ml[idx * 2 + 1];
        num += w * a.part_o[idx * D + d];
    }
    __bf16* out = static_cast<__bf16*>(a.o) + (static_cast<int64_t>(req) * a.Hq + head) * D + d;
    *out = static_cast<__bf16>(num / den);
}

}  // namespace

bool launch_decode_splitk(const DecodeArgs& a, hipStream_t stream) {
    const int group = a.Hq / a.H;
    const int hb_per_kv = (group + 15) / 16;
    const int units = a.H * hb_per_kv;
    const int waves = units < kMaxWaves ? units : kMaxWaves;
    dim3 grid(static_cast<unsigned>(a.total_chunks), static_cast<unsigned>((units + waves - 1) / waves));
    dim3 block(static_cast<unsigned>(waves * 64));
    if (a.D == 128) {
        const size_t lds = static_cast<size_t>(waves) * Geo<128>::WAVE_LDS;
        static bool attr_set = false;
        if (!attr_set) {
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(decode_splitk_kernel<128>), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxWaves * Geo<128>::WAVE_LDS), "hipFuncSetAttribute")) return false;
            attr_set = true;
        }
        hipLaunchKernelGGL(decode_splitk_kernel<128>, grid, block, lds, stream, a, units, hb_per_kv);
    } else {
        const size_t lds = static_cast<size_t>(waves) * Geo<64>::WAVE_LDS;
        static bool attr_set = false;
        if (!attr_set) {
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(decode_splitk_kernel<64>), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxWaves * Geo<64>::WAVE_LDS), "hipFuncSetAttribute")) return false;
            attr_set = true;
        }
        hipLaunchKernelGGL(decode_splitk_kernel<64>, grid, block, lds, stream, a, units, hb_per_kv);
    }
    return hip_ok(hipGetLastError(), "decode split-K launch");
}

bool launch_decode_reduce(const DecodeArgs& a, hipStream_t stream) {
    dim3 grid(static_cast<unsigned>(a.n * a.Hq));
    if (a.D == 128) hipLaunchKernelGGL(decode_reduce_kernel<128>, grid, dim3(128), 0, stream, a);
    else hipLaunchKernelGGL(decode_reduce_kernel<64>, grid, dim3(64), 0, stream, a);
    return hip_ok(hipGetLastError(), "decode reduce launch");
}

}  // namespace vattn
