// Exact merge of partial attentions (per row: weights exp(lse_p - L), L = ln sum_p exp(lse_p)).
// A streaming map bound by HBM bandwidth: every thread owns four consecutive value columns of
// one row, reads them from each of the n partials with one 128-bit load, and writes one
// 128-bit result.  The n log-sum-exps of the row are read by all d/4 threads of the row (one
// cache line broadcast); the first of them also writes the merged lse.
#include <hip/hip_runtime.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

// grid.x covers the 256-thread pieces of a block of RPB rows (RPB * d/4 float4s), grid.y/z the
// row blocks: no thread divides a 64-bit index, and workgroups run through memory in order.
constexpr int MERGE_RPB = 64;

template <int N>   // N > 0: compile-time partial count; N == 0: runtime p.n
__global__ __launch_bounds__(256) void merge_kernel(const MergeParams p, int dq /* d/4 */) {
    const int n = N > 0 ? N : p.n;
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    const unsigned r_in = t / (unsigned)dq;
    const int64_t row = ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * MERGE_RPB + r_in;
    if (r_in >= MERGE_RPB || row >= p.rows) return;
    const unsigned col = t - r_in * dq;
    const int64_t i = row * dq + col;
    float l[16];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < (N > 0 ? N : 16); ++j)
        if (j < n) {
            l[j] = p.lse[j][row];
            m = fmaxf(m, l[j]);
        }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float tot = 0.f;
    const float msafe = (m == -INFINITY) ? 0.f : m;
#pragma unroll
    for (int j = 0; j < (N > 0 ? N : 16); ++j)
        if (j < n) {
            const float w = __expf(l[j] - msafe);      // exp(-inf) = 0 for an empty partial
            if (w > 0.f) {                             // a weight-0 partial is never read
                const float4 x = nt_load4(reinterpret_cast<const float4*>(p.part[j]) + i);
                acc.x += w * x.x; acc.y += w * x.y; acc.z += w * x.z; acc.w += w * x.w;
                tot += w;
            }
        }
    const float inv = tot > 0.f ? 1.0f / tot : 0.f;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    nt_store4(reinterpret_cast<float4*>(p.out) + i, acc);
    if (p.lse_out != nullptr && col == 0)
        p.lse_out[row] = tot > 0.f ? msafe + __logf(tot) : -INFINITY;
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x)
        nt_store4(dst + i, nt_load4(src + i));
}

// One item per thread: a grid of exactly ceil(items / 256) workgroups, dispatched in address order,
// streams through HBM measurably faster than a capped grid whose workgroups stride over the data
// (plain copy of 1.46 GB on MI355X: 6.5 TB/s against 5.1 TB/s with 32 workgroups per CU).  The
// kernels keep their stride loops for grids clipped at the 2^31 - 1 limit of a launch dimension.
static unsigned grid_for(int64_t items) {
    const int64_t blocks = (items + 255) / 256;
    const int64_t cap = 0x7fffffff;
    return (unsigned)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

hipError_t launch_merge(const MergeParams& p, int d, hipStream_t st) {
    const int dq = d / 4;
    const int64_t blocks = (p.rows + MERGE_RPB - 1) / MERGE_RPB;
    const int64_t gy = blocks < 65535 ? blocks : 65535;
    const dim3 g((unsigned)((MERGE_RPB * dq + 255) / 256), (unsigned)gy, (unsigned)((blocks + gy - 1) / gy));
    switch (p.n) {
        case 2: hipLaunchKernelGGL(merge_kernel<2>, g, dim3(256), 0, st, p, dq); break;
        case 3: hipLaunchKernelGGL(merge_kernel<3>, g, dim3(256), 0, st, p, dq); break;
        case 4: hipLaunchKernelGGL(merge_kernel<4>, g, dim3(256), 0, st, p, dq); break;
        case 8: hipLaunchKernelGGL(merge_kernel<8>, g, dim3(256), 0, st, p, dq); break;
        default: hipLaunchKernelGGL(merge_kernel<0>, g, dim3(256), 0, st, p, dq); break;
    }
    return hipGetLastError();
}

hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st) {
    hipLaunchKernelGGL(copy_f32_kernel, dim3(grid_for(n / 4)), dim3(256), 0, st,
                       reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), n / 4);
    return hipGetLastError();
}

}  // namespace pda
