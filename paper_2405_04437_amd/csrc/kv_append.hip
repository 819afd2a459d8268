// KV append: the new K and V rows of every request are copied to the end of its virtually
// contiguous sub-tensor (Sec. 7.1 of the paper: with contiguous KV the append is one plain copy).  Pure data movement:
// 16 bytes per lane, rows are H*D*P bytes and land at consecutive addresses (tok_stride = H*D*P; with
// the all-layers-in-one-buffer layout consecutive tokens of a layer are N*H*D*P apart and each row is
// still one contiguous piece), so both the reads and the writes are fully coalesced.
#include <hip/hip_ext.h>

#include "vattn_internal.h"

namespace vattn {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// grid.x covers 16-byte pieces of the packed new rows; grid.y = 0 for K, 1 for V.
template <bool INL>
__global__ __launch_bounds__(256) void append_kv_kernel(AppendArgs a, InlineMeta im) {
    auto reqid_of = [&](int r) { if constexpr (INL) return im.v[r]; else return a.reqids[r]; };
    auto before_of = [&](int r) { if constexpr (INL) return im.v[a.n + r]; else return a.kv_before[r]; };
    auto cu_of = [&](int r) { if constexpr (INL) return im.v[2 * a.n + r]; else return a.cu_q[r]; };
    const int64_t pieces_per_row = a.row_bytes / 16;
    const int64_t total = static_cast<int64_t>(a.total_rows) * pieces_per_row;
    const char* src = static_cast<const char*>(blockIdx.y == 0 ? a.k_new : a.v_new);
    char* dst_base = blockIdx.y == 0 ? a.k_base : a.v_base;
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int row = static_cast<int>(i / pieces_per_row);
        const int64_t piece = i - static_cast<int64_t>(row) * pieces_per_row;
        // binary search: largest r with cu_q[r] <= row
        int lo = 0, hi = a.n;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cu_of(mid) <= row) lo = mid; else hi = mid;
        }
        const int64_t tok = static_cast<int64_t>(before_of(lo)) + (row - cu_of(lo));
        char* dst = dst_base + static_cast<int64_t>(reqid_of(lo)) * a.S + tok * a.tok_stride + piece * 16;
        *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(src + i * 16);
    }
}

}  // namespace

bool launch_append_kv(const AppendArgs& a, const InlineMeta* im, hipStream_t stream, LaunchEvents ev) {
    if (a.total_rows == 0) return true;
    const int64_t total = static_cast<int64_t>(a.total_rows) * (a.row_bytes / 16);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    dim3 grid(static_cast<unsigned>(blocks), 2);
    static const InlineMeta kNoInline{};
    if (a.inline_meta && im) hipExtLaunchKernelGGL(append_kv_kernel<true>, grid, dim3(256), 0, stream, ev.start, ev.stop, 0, a, *im);
    else hipExtLaunchKernelGGL(append_kv_kernel<false>, grid, dim3(256), 0, stream, ev.start, ev.stop, 0, a, kNoInline);
    return hip_ok(hipGetLastError(), "append_kv launch");
}

}  // namespace vattn
