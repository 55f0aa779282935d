// Data-movement kernels around the attention call, all bound by HBM bandwidth:
//   * postprocess_kernel: Algorithm 1 steps 10-13 (concat, view(-1,h,n,D), permute(0,2,1,3),
//     view(-1,h*n,D)) as ONE pass: hidden[r, i*h + j, :] = chunk_j[r, i, :].
//   * scatter_heads_kernel: the hand-off of a head group into a token-major hidden-state buffer,
//     hidden[s, slot(k), :] = out[k, s, :], with slot(k) either the order in which PipeSP's
//     per-head exchanges deliver the heads (k_mod = j*n + i for k = i*h + j) or the final
//     head-contiguous order (k_orig = k), i.e. with the post-processing folded into the copy.
//   * pack_heads_kernel: token-major fp32 projections -> head-major bf16, optionally dividing
//     every d-vector by its root mean square.
// Every thread moves 16 bytes of fp32; a d-vector (64 or 128 floats) is one 256/512-byte segment,
// so both sides of each copy are made of full cache lines.
#include <hip/hip_runtime.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

static unsigned grid_1d(int64_t items, int64_t cap = 256 * 32) {
    int64_t blocks = (items + 255) / 256;
    return (unsigned)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

// blockIdx.y = local head j (so the chunk pointer is wave-uniform and comes from the kernel
// arguments); blockIdx.x strides over the (row, source GPU i, 4-column) items of that chunk.
__global__ __launch_bounds__(256) void postprocess_kernel(const PostParams p) {
    const int j = blockIdx.y;
    const float4* __restrict__ src = reinterpret_cast<const float4*>(p.chunk[j]);
    float4* __restrict__ dst = reinterpret_cast<float4*>(p.hidden);
    const int64_t per_row = (int64_t)p.n * p.D4;             // float4s of one chunk row
    const int64_t total = p.rows * per_row;
    const int64_t out_row = per_row * p.h;                   // float4s of one hidden row
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = t / per_row;
        const int rem = (int)(t - r * per_row);
        const int i = rem / p.D4;
        const int c = rem - i * p.D4;
        nt_store4(dst + r * out_row + (int64_t)(i * p.h + j) * p.D4 + c, nt_load4(src + r * p.row_stride4 + rem));
    }
}

hipError_t launch_postprocess(const PostParams& p, hipStream_t st) {
    const int64_t per_chunk = p.rows * p.n * p.D4;
    const unsigned gx = grid_1d(per_chunk, (256 * 32 + p.h - 1) / p.h);
    hipLaunchKernelGGL(postprocess_kernel, dim3(gx, p.h), dim3(256), 0, st, p);
    return hipGetLastError();
}

// src: hg heads of one batch, [hg, S, d] contiguous (heads h0 .. h0+hg-1 of the full H = n*h);
// dst: that batch's [S, H, d].
__global__ __launch_bounds__(256) void scatter_heads_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                            int64_t S, int d4, int hg, int H, int h0, int h, int n,
                                                            int arrival) {
    const int64_t per_head = S * d4;
    const int64_t total = per_head * hg;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int jj = (int)(t / per_head);
        const int64_t rem = t - (int64_t)jj * per_head;
        const int64_t s = rem / d4;
        const int c = (int)(rem - s * d4);
        const int k = h0 + jj;                               // global head = i*h + j
        const int slot = arrival ? (k % h) * n + k / h : k;  // k_mod(i,j) = j*n + i, or k_orig
        nt_store4(dst + (s * H + slot) * d4 + c, nt_load4(src + t));
    }
}

hipError_t launch_scatter_heads(const float* src, float* dst, int64_t S, int d, int hg, int H, int h0,
                                int h, int n, int arrival, hipStream_t st) {
    hipLaunchKernelGGL(scatter_heads_kernel, dim3(grid_1d((int64_t)hg * S * (d / 4))), dim3(256), 0, st,
                       reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), S, d / 4, hg, H, h0, h, n, arrival);
    return hipGetLastError();
}

// LPV = lanes per d-vector (d/4: 16 or 32).  Items are ordered by OUTPUT position, so the bf16
// writes are contiguous and the fp32 reads are d-float segments H*d floats apart.
template <int LPV>
__global__ __launch_bounds__(256) void pack_heads_kernel(const float4* __restrict__ x, uint2* __restrict__ y,
                                                         int64_t S, int H, int64_t n_vec /* B*H*S */, int unit_rms, float premul) {
    constexpr int VPB = 256 / LPV;                            // vectors per workgroup pass
    const int lane = threadIdx.x % LPV;
    const int64_t n_pass = (n_vec + VPB - 1) / VPB;
    for (int64_t pass = blockIdx.x; pass < n_pass; pass += gridDim.x) {
        const int64_t o = pass * VPB + threadIdx.x / LPV;     // output vector index (b*H + h)*S + s
        const bool live = o < n_vec;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live) {
            const int64_t bh = o / S;
            const int64_t s = o - bh * S;
            const int64_t b = bh / H;
            const int hh = (int)(bh - b * H);
            a = nt_load4(x + ((b * S + s) * H + hh) * LPV + lane);
        }
        if (unit_rms) {
            float ss = a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
#pragma unroll
            for (int m = 1; m < LPV; m <<= 1) ss += __shfl_xor(ss, m, LPV);
            const float inv = ss > 0.f ? premul / sqrtf(ss * (1.0f / (4 * LPV))) : 0.f;
            a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
        } else if (premul != 1.0f) {
            a.x *= premul; a.y *= premul; a.z *= premul; a.w *= premul;
        }
        if (live) {
            nt_store2(y + o * LPV + lane, pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));   // round to nearest even
        }
    }
}

hipError_t launch_pack(const float* x, void* y, int B, int64_t S, int H, int d, int unit_rms, float premul, hipStream_t st) {
    const int64_t n_vec = (int64_t)B * H * S;
    const float4* xs = reinterpret_cast<const float4*>(x);
    uint2* yd = reinterpret_cast<uint2*>(y);
    if (d == 128) {
        hipLaunchKernelGGL(pack_heads_kernel<32>, dim3(grid_1d(n_vec * 32)), dim3(256), 0, st, xs, yd, S, H, n_vec, unit_rms, premul);
    } else {
        hipLaunchKernelGGL(pack_heads_kernel<16>, dim3(grid_1d(n_vec * 16)), dim3(256), 0, st, xs, yd, S, H, n_vec, unit_rms, premul);
    }
    return hipGetLastError();
}

}  // namespace pda
