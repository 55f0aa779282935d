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

// Launch shape of the streaming kernels here.  One item per thread, workgroups dispatched in
// address order: a grid of exactly as many workgroups as there are items streams through HBM
// measurably faster than a capped grid whose workgroups stride over the data.  Long axes (rows,
// tokens) are spread over grid.y and grid.z so that no thread divides a 64-bit index (a 64-bit
// division costs about a hundred instructions per thread, more than the copy itself).
struct RowGrid {
    unsigned y, z;
};
static RowGrid row_grid(int64_t rows) {
    const int64_t y = rows < 65535 ? (rows > 0 ? rows : 1) : 65535;
    return {(unsigned)y, (unsigned)((rows + y - 1) / y)};     // up to 65535^2 rows
}
__device__ __forceinline__ int64_t grid_row() { return (int64_t)blockIdx.z * gridDim.y + blockIdx.y; }

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xF, 0xF, false));
}

// Algorithm 1 steps 10-13.  grid.y/z = row r; grid.x covers the row's h*n*D/4 float4s in INPUT
// order of the concatenated tensor (local head j, source GPU i, 4 columns): consecutive
// workgroups read consecutive memory when the chunks are the slices of one concatenated
// [rows, h*n, D] tensor (h sequential streams when they are separate tensors) and write inside
// the same hidden row.  The chunk pointers are read from the kernel arguments with a per-lane
// index (uniform over a wavefront whenever n*D/4 is a multiple of 64).
__global__ __launch_bounds__(256) void postprocess_kernel(const PostParams p) {
    const int64_t r = grid_row();
    const unsigned per_row = (unsigned)p.n * p.D4;           // float4s of one chunk row
    const unsigned out_row = per_row * p.h;                  // float4s of one hidden row
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    if (r >= p.rows || t >= out_row) return;
    const unsigned j = t / per_row;
    const unsigned rem = t - j * per_row;
    const unsigned i = rem / (unsigned)p.D4;
    const unsigned c = rem - i * p.D4;
    const float4* __restrict__ src = reinterpret_cast<const float4*>(p.chunk[j]);
    float4* __restrict__ dst = reinterpret_cast<float4*>(p.hidden);
    nt_store4(dst + r * out_row + (i * p.h + j) * p.D4 + c, nt_load4(src + r * p.row_stride4 + rem));
}

hipError_t launch_postprocess(const PostParams& p, hipStream_t st) {
    const RowGrid g = row_grid(p.rows);
    const unsigned out_row = (unsigned)p.n * p.D4 * p.h;
    hipLaunchKernelGGL(postprocess_kernel, dim3((out_row + 255) / 256, g.y, g.z), dim3(256), 0, st, p);
    return hipGetLastError();
}

// src: hg heads of one batch, [hg, S, d] contiguous (heads h0 .. h0+hg-1 of the full H = n*h);
// dst: that batch's [S, H, d].  grid.y/z = block of TOK tokens; grid.x covers the block's
// TOK*hg*d/4 float4s in OUTPUT order (token, head of the group, 4 columns): the group's heads of
// one token are written next to each other where their slots are adjacent; reads are hg
// sequential streams.
constexpr int SCATTER_TOK = 64;
__global__ __launch_bounds__(256) void scatter_heads_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                            int64_t S, int d4, int hg, int H, int h0, int h, int n,
                                                            int arrival) {
    const unsigned per_tok = (unsigned)hg * d4;
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    const unsigned tok = t / per_tok;
    const int64_t s = grid_row() * SCATTER_TOK + tok;
    if (tok >= SCATTER_TOK || s >= S) return;
    const unsigned rem = t - tok * per_tok;
    const unsigned jj = rem / (unsigned)d4;
    const unsigned c = rem - jj * d4;
    const int k = h0 + (int)jj;                              // global head = i*h + j
    const int slot = arrival ? (k % h) * n + k / h : k;      // k_mod(i,j) = j*n + i, or k_orig
    nt_store4(dst + (s * H + slot) * d4 + c, nt_load4(src + (int64_t)jj * S * d4 + s * d4 + c));
}

hipError_t launch_scatter_heads(const float* src, float* dst, int64_t S, int d, int hg, int H, int h0,
                                int h, int n, int arrival, hipStream_t st) {
    const RowGrid g = row_grid((S + SCATTER_TOK - 1) / SCATTER_TOK);
    const unsigned items = (unsigned)SCATTER_TOK * hg * (d / 4);
    hipLaunchKernelGGL(scatter_heads_kernel, dim3((items + 255) / 256, g.y, g.z), dim3(256), 0, st,
                       reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), S, d / 4, hg, H, h0, h, n, arrival);
    return hipGetLastError();
}

// LPV = lanes per d-vector (d/4: 16 or 32).  A workgroup packs VPB consecutive tokens of one head:
// it reads VPB d-float segments (H*d floats apart) and writes VPB*d contiguous bf16.
// grid.x = head, grid.y/z = (batch, token block): the H workgroups of one token block, dispatched
// one after the other, together read one contiguous piece of x, and every head's output advances
// sequentially.
template <int LPV>
__global__ __launch_bounds__(256) void pack_heads_kernel(const float4* __restrict__ x, uint2* __restrict__ y,
                                                         int64_t S, int H, int64_t n_blk /* ceil(S/VPB) */, int B,
                                                         int unit_rms, float premul) {
    constexpr int VPB = 256 / LPV;                            // tokens per workgroup
    const int lane = threadIdx.x % LPV;
    const int hh = blockIdx.x;
    const int64_t bb = grid_row();                            // b * n_blk + block
    if (bb >= n_blk * B) return;
    int64_t b = 0, blk = bb;
    if (B > 1) { b = bb / n_blk; blk = bb - b * n_blk; }     // wave-uniform, taken only with several batches
    const int64_t s = blk * VPB + threadIdx.x / LPV;
    const bool live = s < S;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) a = nt_load4(x + ((b * S + s) * H + hh) * LPV + lane);
    if (unit_rms) {
        // sum of squares over the vector's LPV lanes, in registers (DPP lane permutations and, for
        // 32 lanes, the 16-lane row swap): every lane ends up with the total
        float ss = a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        ss += dpp_f32<0xB1>(ss);          // quad_perm [1,0,3,2]: lane ^ 1
        ss += dpp_f32<0x4E>(ss);          // quad_perm [2,3,0,1]: lane ^ 2
        ss += dpp_f32<0x141>(ss);         // row_half_mirror: the other quad of each 8
        ss += dpp_f32<0x140>(ss);         // row_mirror: the other half of each 16
        if constexpr (LPV == 32) {
            auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(ss), __float_as_uint(ss), false, false);
            ss = __uint_as_float(r[0]) + __uint_as_float(r[1]);    // lane ^ 16
        }
        // 1/sqrt by the hardware approximation (1 ulp): far inside the bf16 rounding that follows
        const float inv = ss > 0.f ? premul * __builtin_amdgcn_rsqf(ss * (1.0f / (4 * LPV))) : 0.f;
        a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
    } else if (premul != 1.0f) {
        a.x *= premul; a.y *= premul; a.z *= premul; a.w *= premul;
    }
    if (live) {
        nt_store2(y + ((b * H + hh) * S + s) * LPV + lane, pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));   // round to nearest even
    }
}

hipError_t launch_pack(const float* x, void* y, int B, int64_t S, int H, int d, int unit_rms, float premul, hipStream_t st) {
    const float4* xs = reinterpret_cast<const float4*>(x);
    uint2* yd = reinterpret_cast<uint2*>(y);
    const int vpb = d == 128 ? 8 : 16;
    const int64_t n_blk = (S + vpb - 1) / vpb;
    const RowGrid g = row_grid(n_blk * B);
    if (d == 128) {
        hipLaunchKernelGGL(pack_heads_kernel<32>, dim3(H, g.y, g.z), dim3(256), 0, st, xs, yd, S, H, n_blk, B, unit_rms, premul);
    } else {
        hipLaunchKernelGGL(pack_heads_kernel<16>, dim3(H, g.y, g.z), dim3(256), 0, st, xs, yd, S, H, n_blk, B, unit_rms, premul);
    }
    return hipGetLastError();
}

}  // namespace pda
