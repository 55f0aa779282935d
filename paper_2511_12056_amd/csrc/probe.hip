// Matrix-pipe rate probe: a loop of nothing but v_mfma_f32_32x32x16_bf16 on operand fragments
// read once from a caller-supplied bf16 buffer.  The rate this device sustains depends on the
// operand DATA (the chip lowers its clock under the switching activity of random mantissas), so
// the probe is run on the same tensors as the attention kernel to say what the matrix pipe alone
// can do on them.
#include <hip/hip_runtime.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

// 8 wavefronts per workgroup (two per SIMD), one workgroup per CU; every lane keeps 8 A and 8 B
// fragments in registers and cycles through them with four independent accumulators.
__global__ __launch_bounds__(512, 1) void mfma_rate_kernel(const bf16x8* __restrict__ src, int64_t n_frag,
                                                           int64_t iters, float* __restrict__ sink) {
    bf16x8 a[8], b[8];
    const int64_t base = ((int64_t)blockIdx.x * 512 + threadIdx.x) * 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = src[(base + i) % n_frag];
        b[i] = src[(base + 8 + i) % n_frag];
    }
    f32x16 c0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; j += 4) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j + 1], b[j + 1], c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j + 2], b[j + 2], c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j + 3], b[j + 3], c3, 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    // keeps the loop alive; one float per lane of the first workgroup is enough
    if (blockIdx.x == 0) sink[threadIdx.x] = s;
}

hipError_t launch_mfma_rate(const void* src, int64_t n_frag, int64_t iters, int n_cu, float* sink, hipStream_t st) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(n_cu), dim3(512), 0, st, static_cast<const bf16x8*>(src), n_frag, iters, sink);
    return hipGetLastError();
}

}  // namespace pda
