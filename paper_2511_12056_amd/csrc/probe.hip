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

// The same loop with the other instruction classes of the attention kernel's inner loop added, at
// the kernel's own density per MFMA, so that their cost under the chip's power limit can be read
// off one after the other on the caller's data:
//   MIX 1: + the softmax arithmetic (per MFMA: one v_fma_f32, one v_exp_f32, one v_add_f32, half a
//            v_cvt_pk_bf16_f32), fed from the accumulators
//   MIX 2: + the MFMA A operands read from LDS as the kernel reads them (per two MFMAs: one
//            ds_read_b128 and one pair of transposing ds_read_b64_tr_b16), LDS filled from src
//   MIX 3: MIX 2 with the reads a wavefront owning 64 instead of 32 query rows would need (every
//            operand fragment feeds two MFMAs: half the reads)
// No global->LDS traffic, no barriers, no dependencies between the classes: an upper bound for
// the kernel's steady state, not a model of it.
template <int MIX>
__global__ __launch_bounds__(512, 1) void loop_mix_kernel(const bf16x8* __restrict__ src, int64_t n_frag,
                                                          int64_t iters, float* __restrict__ sink) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];      // 64 KB
    bf16x8 a[4], b[8];
    const int64_t base = ((int64_t)blockIdx.x * 512 + threadIdx.x) * 12;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = src[(base + i) % n_frag];
#pragma unroll
    for (int i = 0; i < 8; ++i) b[i] = src[(base + 4 + i) % n_frag];
    for (int i = threadIdx.x; i < 4096; i += 512) reinterpret_cast<bf16x8*>(smem)[i] = src[((int64_t)blockIdx.x * 4096 + i) % n_frag];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    // every wavefront reads its own 8 KB; 16-byte reads at lane*16 and 8-byte transposing reads at lane*8 are conflict free
    LDS_PTR(const unsigned char) lp = (LDS_PTR(const unsigned char))smem + (threadIdx.x >> 6) * 8192;
    f32x16 c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    float sum = 0.f;
    unsigned pk = 0u;
    float zs[16], es[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) { zs[i] = 0.f; es[i] = 0.f; }
    // operand fragments are read three MFMAs ahead of their use (a ring of four), as in the kernel
    bf16x8 fr[4] = {a[0], a[1], a[2], a[3]};
    auto read_frag = [&](auto uc) {
        constexpr int u = decltype(uc)::value % 16;
        constexpr bool rd = MIX == 2 || (MIX == 3 && u % 2 == 0);
        if constexpr (rd && (MIX == 2 ? u % 2 == 0 : u % 4 == 0)) {
            fr[u % 4] = *(LDS_PTR(const bf16x8))(lp + lane * 16 + (u / 2) * 1024);
        } else if constexpr (rd) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(lp + lane * 8 + (u / 2) * 1024));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(lp + lane * 8 + (u / 2) * 1024 + 512));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            fr[u % 4] = __builtin_bit_cast(bf16x8, av);
        }
    };
    read_frag(std::integral_constant<int, 0>{});
    read_frag(std::integral_constant<int, 1>{});
    read_frag(std::integral_constant<int, 2>{});
    for (int64_t it = 0; it < iters; ++it) {
        static_for<0, 16>([&](auto uc) {                  // 16 MFMAs per iteration
            constexpr int u = decltype(uc)::value;
            const bf16x8 A = fr[u % 4];
            c[u % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, b[u % 8], c[u % 4], 0, 0, 0);
            read_frag(std::integral_constant<int, u + 3>{});
            if constexpr (MIX >= 1) {
                // one score per MFMA: scale-and-shift, exponential, add to the row sum; a pack every other MFMA.
                // Each step reads what an earlier unit produced, as in the kernel.
                float z = __builtin_fmaf(c[(u + 1) % 4][u], 1e-4f, -1.0f);   // an accumulator last written three MFMAs ago
                asm volatile("" : "+v"(z));
                float e = __builtin_amdgcn_exp2f(zs[(u + 15) % 16]);
                asm volatile("" : "+v"(e));
                sum += es[(u + 14) % 16];
                asm volatile("" : "+v"(sum));
                if (u % 2 == 0) {
                    unsigned h = pack_bf16(es[(u + 12) % 16], es[(u + 13) % 16]);
                    asm volatile("" : "+v"(h));
                    pk ^= h;
                }
                zs[u] = z;
                es[u] = e;
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    float s = sum + (float)(pk & 0xffu);
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[0][r] + c[1][r] + c[2][r] + c[3][r];
    if (blockIdx.x == 0) sink[threadIdx.x] = s;
}

hipError_t launch_mfma_rate(const void* src, int64_t n_frag, int64_t iters, int n_cu, int mix, float* sink, hipStream_t st) {
    const bf16x8* p = static_cast<const bf16x8*>(src);
    constexpr int smem = 65536;
    if (mix == 0) {
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(n_cu), dim3(512), 0, st, p, n_frag, iters, sink);
        return hipGetLastError();
    }
    static KernelSetup s1, s2, s3;
    hipError_t e = hipSuccess;
    const int64_t it16 = (iters + 1) / 2;            // 16 MFMAs per iteration here, 8 in the MFMA-only loop
    switch (mix) {
        case 1:
            if ((e = s1.ensure(reinterpret_cast<const void*>(loop_mix_kernel<1>), smem, nullptr)) != hipSuccess) return e;
            hipLaunchKernelGGL(loop_mix_kernel<1>, dim3(n_cu), dim3(512), smem, st, p, n_frag, it16, sink);
            break;
        case 2:
            if ((e = s2.ensure(reinterpret_cast<const void*>(loop_mix_kernel<2>), smem, nullptr)) != hipSuccess) return e;
            hipLaunchKernelGGL(loop_mix_kernel<2>, dim3(n_cu), dim3(512), smem, st, p, n_frag, it16, sink);
            break;
        default:
            if ((e = s3.ensure(reinterpret_cast<const void*>(loop_mix_kernel<3>), smem, nullptr)) != hipSuccess) return e;
            hipLaunchKernelGGL(loop_mix_kernel<3>, dim3(n_cu), dim3(512), smem, st, p, n_frag, it16, sink);
            break;
    }
    return hipGetLastError();
}

}  // namespace pda
