// Micro-benchmarks of the two roofs.  Matrix pipes: what dense bf16 rate the chip sustains with nothing else going on.
//
// Every wave runs rounds of four independent v_mfma_f32_32x32x16_bf16 whose operands stay in registers
// (no LDS, no memory traffic inside the timed loop), two waves per SIMD on every CU.  With all-zero
// operands the chip holds its full clock; with N(0,1) operands - the distribution of the attention
// workloads here - it lowers the clock to stay inside its power limit, which sets the rate a bf16
// contraction over such data can reach at best.  The shader clock is read off inside the kernel as
// the ratio of the shader-cycle counter to the constant 100 MHz counter.  Optionally every matrix instruction is
// accompanied by the side work of an attention inner loop (an operand read from LDS, fp32 multiply-adds, an
// exp2), which shows what each of them costs once the power limit sets the clock.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "vattn_internal.h"

namespace vattn {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kChains = 4;           // independent accumulators per wave
constexpr int kWavesPerGroup = 4;

// src: 2 * kChains operand vectors of 64 lanes x 16 B, shared by all waves.
// SIDE adds, per matrix instruction, the other work an attention inner loop does beside it - so that its cost under
// the chip's power limit can be read off one by one: bit 0 = the A operand comes from LDS (one 16-byte read per lane
// and instruction, fetched a round ahead), bit 1 = three independent fp32 multiply-adds, bit 2 = one exp2.
constexpr int kProbeLds = 32 * 1024;
template <int SIDE>
__global__ __launch_bounds__(kWavesPerGroup * 64) void mfma_loop_kernel(const u32x4* src, float* sink, int rounds,
                                                                          unsigned long long* clocks) {
    __shared__ __attribute__((aligned(16))) char lds[(SIDE & 1) ? kProbeLds : 16];
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
    if constexpr (SIDE & 1) {
        for (int i = threadIdx.x; i < kProbeLds / 16; i += kWavesPerGroup * 64) reinterpret_cast<u32x4*>(lds)[i] = src[i % (2 * kChains * 64)];
        __syncthreads();
    }
    bf16x8 a[kChains], a2[kChains], b[kChains];
    f32x16 acc[kChains];
#pragma unroll
    for (int j = 0; j < kChains; ++j) {
        a[j] = a2[j] = __builtin_bit_cast(bf16x8, src[j * 64 + l]);
        b[j] = __builtin_bit_cast(bf16x8, src[(kChains + j) * 64 + l]);
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    }
    float v[3] = {0.001f * l, 0.002f * l, 0.003f * l}, e = 0.5f + 0.001f * l;
    int off = w * 8192;
    auto fetch = [&](bf16x8 (&dst)[kChains], int o) {
        if constexpr (SIDE & 1) {
#pragma unroll
            for (int j = 0; j < kChains; ++j) dst[j] = *reinterpret_cast<const bf16x8*>(lds + ((o + j * 1024 + l * 16) & (kProbeLds - 1)));
        }
    };
    auto work = [&](const bf16x8 (&aa)[kChains]) {
#pragma unroll
        for (int j = 0; j < kChains; ++j) {
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aa[j], b[j], acc[j], 0, 0, 0);
            if constexpr (SIDE & 2) {
#pragma unroll
                for (int i = 0; i < 3; ++i) v[i] = __builtin_fmaf(v[i], 1.0001f, 0.25f);
            }
            if constexpr (SIDE & 4) e = __builtin_amdgcn_exp2f(e) * 0.5f;
        }
    };
    fetch(a, off);
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < rounds; it += 2) {
        fetch(a2, off + 4096);
        work(a);
        fetch(a, off + 8192);
        work(a2);
        off = (off + 8192) & (kProbeLds - 1);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = e + v[0] + v[1] + v[2];
#pragma unroll
    for (int j = 0; j < kChains; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0) { clocks[blockIdx.x * 2] = c1 - c0; clocks[blockIdx.x * 2 + 1] = w1 - w0; }
}

// Streaming-read micro-benchmark: what HBM delivers to a kernel that only reads.  One workgroup of four waves per
// CU walks its own contiguous share of the buffer with 16-byte non-temporal loads, 16 per lane in flight - the
// launch shape and load pattern of the decode kernel without its arithmetic.
constexpr int kStreamUnroll = 16;
__global__ __launch_bounds__(kWavesPerGroup * 64) void stream_read_kernel(const u32x4* src, size_t vec_per_group, uint32_t* sink) {
    const u32x4* p = src + static_cast<size_t>(blockIdx.x) * vec_per_group + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    const size_t rounds = vec_per_group / (kWavesPerGroup * 64 * kStreamUnroll);
    for (size_t r = 0; r < rounds; ++r) {
        u32x4 v[kStreamUnroll];
#pragma unroll
        for (int i = 0; i < kStreamUnroll; ++i) v[i] = __builtin_nontemporal_load(p + static_cast<size_t>(i) * kWavesPerGroup * 64);
#pragma unroll
        for (int i = 0; i < kStreamUnroll; ++i) acc ^= v[i];
        p += static_cast<size_t>(kStreamUnroll) * kWavesPerGroup * 64;
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[blockIdx.x] = acc[0];   // keeps the loads alive; practically never taken
}

}  // namespace

bool stream_microbench(int device, int64_t bytes, double* gbs) {
    if (bytes < (64 << 20) || bytes > (int64_t{64} << 30) || !gbs) { set_error("stream_microbench: size must be between 64 MiB and 64 GiB"); return false; }
    if (!hip_ok(hipSetDevice(device), "hipSetDevice")) return false;
    int cus = 0;
    if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device), "hipDeviceGetAttribute")) return false;
    const size_t round_vecs = static_cast<size_t>(kWavesPerGroup) * 64 * kStreamUnroll;                 // 16-byte vectors per round
    const size_t vec_per_group = static_cast<size_t>(bytes) / 16 / static_cast<size_t>(cus) / round_vecs * round_vecs;
    const size_t total = vec_per_group * static_cast<size_t>(cus) * 16;
    u32x4* buf = nullptr; uint32_t* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = hip_ok(hipMalloc(reinterpret_cast<void**>(&buf), total), "hipMalloc") &&
              hip_ok(hipMalloc(reinterpret_cast<void**>(&sink), static_cast<size_t>(cus) * 4), "hipMalloc") &&
              hip_ok(hipMemset(buf, 0x5A, total), "hipMemset") &&
              hip_ok(hipEventCreate(&e0), "hipEventCreate") && hip_ok(hipEventCreate(&e1), "hipEventCreate");
    float best = 0.f;
    for (int rep = 0; ok && rep < 4; ++rep) {   // the first launch warms up; the best of the rest counts
        ok = hip_ok(hipEventRecord(e0, nullptr), "hipEventRecord");
        if (!ok) break;
        stream_read_kernel<<<cus, kWavesPerGroup * 64>>>(buf, vec_per_group, sink);
        float ms = 0.f;
        ok = hip_ok(hipEventRecord(e1, nullptr), "hipEventRecord") && hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize") &&
             hip_ok(hipGetLastError(), "stream_read_kernel") && hip_ok(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime");
        if (ok && rep > 0 && (best == 0.f || ms < best)) best = ms;
    }
    if (ok) *gbs = static_cast<double>(total) / (static_cast<double>(best) * 1e6);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    if (sink) (void)hipFree(sink);
    return ok;
}

bool mfma_microbench(int device, int mode, int rounds, double* tflops, double* shader_mhz) {
    const bool normal_operands = (mode & 1) != 0;
    const int side = (mode >> 1) & 7;
    if (mode < 0 || mode > 15 || rounds < 1 || rounds > 10000000 || !tflops || !shader_mhz) { set_error("mfma_microbench: invalid argument"); return false; }
    if (!hip_ok(hipSetDevice(device), "hipSetDevice")) return false;
    int cus = 0;
    if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device), "hipDeviceGetAttribute")) return false;
    const int groups = cus * 2;   // 8 waves per CU, two per SIMD
    // operands: bf16 bit patterns, N(0,1) from a fixed-seed Box-Muller over a 64-bit LCG, or zeros
    std::vector<uint16_t> h(static_cast<size_t>(2 * kChains) * 64 * 8, 0);
    if (normal_operands) {
        uint64_t st = 0x9E3779B97F4A7C15ull;
        auto uni = [&]() { st = st * 6364136223846793005ull + 1442695040888963407ull; return (static_cast<double>(st >> 11) + 0.5) / 9007199254740992.0; };
        for (auto& x : h) {
            const float f = static_cast<float>(std::sqrt(-2.0 * std::log(uni())) * std::cos(6.283185307179586 * uni()));
            uint32_t u;
            std::memcpy(&u, &f, 4);
            x = static_cast<uint16_t>((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
        }
    }
    u32x4* src = nullptr; float* sink = nullptr; unsigned long long* clocks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = hip_ok(hipMalloc(reinterpret_cast<void**>(&src), h.size() * 2), "hipMalloc") &&
              hip_ok(hipMalloc(reinterpret_cast<void**>(&sink), static_cast<size_t>(groups) * kWavesPerGroup * 64 * 4), "hipMalloc") &&
              hip_ok(hipMalloc(reinterpret_cast<void**>(&clocks), static_cast<size_t>(groups) * 16), "hipMalloc") &&
              hip_ok(hipMemcpy(src, h.data(), h.size() * 2, hipMemcpyHostToDevice), "hipMemcpy") &&
              hip_ok(hipEventCreate(&e0), "hipEventCreate") && hip_ok(hipEventCreate(&e1), "hipEventCreate");
    float ms = 0.f;
    std::vector<unsigned long long> hc(static_cast<size_t>(groups) * 2);
    if (ok) {
        auto launch = [&]() {
            const dim3 g(static_cast<unsigned>(groups)), t(kWavesPerGroup * 64);
            switch (side) {
                case 0: mfma_loop_kernel<0><<<g, t>>>(src, sink, rounds, clocks); break;
                case 1: mfma_loop_kernel<1><<<g, t>>>(src, sink, rounds, clocks); break;
                case 2: mfma_loop_kernel<2><<<g, t>>>(src, sink, rounds, clocks); break;
                case 3: mfma_loop_kernel<3><<<g, t>>>(src, sink, rounds, clocks); break;
                case 4: mfma_loop_kernel<4><<<g, t>>>(src, sink, rounds, clocks); break;
                case 5: mfma_loop_kernel<5><<<g, t>>>(src, sink, rounds, clocks); break;
                case 6: mfma_loop_kernel<6><<<g, t>>>(src, sink, rounds, clocks); break;
                default: mfma_loop_kernel<7><<<g, t>>>(src, sink, rounds, clocks); break;
            }
        };
        // one untimed launch of the same length lets the clock settle where the power limit puts it
        launch();
        ok = hip_ok(hipEventRecord(e0, nullptr), "hipEventRecord");
        if (ok) {
            launch();
            ok = hip_ok(hipEventRecord(e1, nullptr), "hipEventRecord") && hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize") &&
                 hip_ok(hipGetLastError(), "mfma_loop_kernel") && hip_ok(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime") &&
                 hip_ok(hipMemcpy(hc.data(), clocks, hc.size() * 8, hipMemcpyDeviceToHost), "hipMemcpy");
        }
    }
    if (ok) {
        double cyc = 0, wall = 0;
        for (int i = 0; i < groups; ++i) { cyc += static_cast<double>(hc[2 * i]); wall += static_cast<double>(hc[2 * i + 1]); }
        const double flops = static_cast<double>(groups) * kWavesPerGroup * ((rounds + 1) / 2 * 2) * kChains * (2.0 * 32 * 32 * 16);
        *tflops = flops / (static_cast<double>(ms) * 1e9);
        *shader_mhz = wall > 0 ? cyc / wall * 100.0 : 0.0;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (src) (void)hipFree(src);
    if (sink) (void)hipFree(sink);
    if (clocks) (void)hipFree(clocks);
    return ok;
}

}  // namespace vattn
