// Flash-attention forward for gfx950 (MI355X): the per-head attention call of PipeSP's loop
// (Algorithm 1, step 3) and of Attention Co-processing (Attn(Q,K,V)), evaluated tile by tile
// with an online softmax so that the score matrix never leaves the CU.
//
// Work decomposition
//   grid.x = query tiles of M = 32*NQ*NW rows, grid.y = (batch, head) pairs.
//   A workgroup has NW wavefronts; each wavefront owns NQ sub-tiles of 32 query rows and walks
//   all valid keys in steps of BN, reading K/V tiles that the whole workgroup stages in LDS
//   (double-buffered: the global loads of tile t+1 are in flight while tile t is consumed).
//
// Matrix-core formulation (v_mfma_f32_32x32x16_bf16, A 32x16, B 16x32, D 32x32):
//   S^T = K Q^T    A = K tile rows (lane: key l%32, 8 consecutive d at 8*(l/32)), read from LDS
//                  B = Q^T (lane: query l%32, same 8 d), held in registers for the whole sweep
//                  D: lane holds ONE query (l%32) and 16 keys 8a+4(l/32)+b  (register r = 4a+b)
//   O^T = V^T P^T  A = V^T (lane: value column l%32, 8 key slots), transposing LDS read
//                  B = P^T (lane: query l%32, 8 key slots) = the lane's own exp'ed S registers
//                  D: lane holds the same query and 16 value columns
// The contraction index of the second product is permuted consistently on both operands so that
// the probabilities feed the second product straight from the registers the first one wrote:
// key slot e (0..7) of half-wave h in the MFMA covering keys [16u, 16u+16) of a 32-key block is
// key 16u + 8(e/4) + 4h + e%4.  Because a lane holds a single query, the running max m, the
// running sum l and the rescale factor are lane-local; the only cross-lane step per tile is one
// swap of the row max between lanes l and l^32.
//
// LDS layout: a tile is BN rows of D bf16 (row = one key), split in 16-byte granules; granule g
// of row r is stored at granule position  g ^ (r % G)  for K (G granules per row) so the
// 128-bit operand reads of 16 consecutive rows hit 16 different bank groups, and at
// g ^ (4*(r%4)) for V so the 4-row transposing reads do.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

template <int D, int NQ, int NW, int BN, int MINB>
__global__ __launch_bounds__(64 * NW, MINB) void attn_fwd_kernel(const AttnParams p) {
    constexpr int T = 64 * NW;            // threads
    constexpr int M = 32 * NQ * NW;       // query rows per workgroup
    constexpr int G = D / 8;              // 16-byte granules per row
    constexpr int NKB = BN / 32;          // 32-key blocks per tile
    constexpr int NKK = D / 16;           // contraction steps of the first product
    constexpr int NDB = D / 32;           // 32-column blocks of the output
    constexpr int NLD = BN * G / T;       // granules each thread stages per tensor per tile
    constexpr int TILE_BYTES = BN * D * 2;
    static_assert(BN * G % T == 0, "tile must divide over the threads");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* const k_lds = smem;                       // [2][BN][D] bf16
    unsigned char* const v_lds = smem + 2 * TILE_BYTES;      // [2][BN][D] bf16

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;

    const int bh = blockIdx.y;
    const int b = bh / p.Hg, h = bh - b * p.Hg;
    const __bf16* __restrict__ qp = p.q + (int64_t)b * p.q_bs + (int64_t)h * p.q_hs;
    const __bf16* __restrict__ kp = p.k + (int64_t)b * p.kv_bs + (int64_t)h * p.kv_hs;
    const __bf16* __restrict__ vp = p.v + (int64_t)b * p.kv_bs + (int64_t)h * p.kv_hs;
    float* __restrict__ op = p.out + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs;
    float* __restrict__ lp = p.lse + (int64_t)b * p.l_bs + (int64_t)h * p.l_hs;

    const int64_t Sq = p.Sq;
    const int n_v = (int)p.n_v;                       // valid keys, >= 1 here
    const int nt = (n_v + BN - 1) / BN;
    const int64_t q_row0 = (int64_t)blockIdx.x * M + wave * (32 * NQ);

    // ---- Q operand fragments, resident for the whole sweep
    bf16x8 qf[NQ][NKK];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        int64_t row = q_row0 + nq * 32 + li;
        row = row < Sq ? row : Sq - 1;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            qf[nq][kk] = *reinterpret_cast<const bf16x8*>(qp + row * D + kk * 16 + 8 * lh);
    }

    // ---- staging of K/V tiles: thread -> (row, granule) of the tile, fixed for all tiles
    u32x4 kreg[NLD], vreg[NLD];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int gid = i * T + tid;
            const int r = gid / G, g = gid % G;
            int row = t * BN + r;
            row = row < n_v ? row : n_v - 1;          // hidden / out-of-range keys are never read
            const int64_t off = (int64_t)row * D + g * 8;
            kreg[i] = *reinterpret_cast<const u32x4*>(kp + off);
            vreg[i] = *reinterpret_cast<const u32x4*>(vp + off);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int gid = i * T + tid;
            const int r = gid / G, g = gid % G;
            const int gk = g ^ (r & (G - 1));
            const int gv = g ^ (((r & 3) << 2) & (G - 1));
            *reinterpret_cast<u32x4*>(k_lds + buf * TILE_BYTES + r * (D * 2) + gk * 16) = kreg[i];
            *reinterpret_cast<u32x4*>(v_lds + buf * TILE_BYTES + r * (D * 2) + gv * 16) = vreg[i];
        }
    };

    // ---- per-lane read offsets
    // K operand: row kb*32+li, granule (2kk+lh) ^ (li % G)
    const int k_row_off = li * (D * 2);
    // V^T operand through the transposing read: within a 16-lane block, lane t supplies the
    // address of 4 consecutive columns (t%4) of key row (t/4) and receives column t of 4 rows.
    const int t16 = lane & 15;
    const int v_key_in = 4 * lh + (t16 >> 2);                  // key inside a 16-key group (first 4-key read)
    const int v_colg = 2 * (li >> 4) + ((t16 & 3) >> 1);       // granule inside a 32-column block
    const int v_sub = (t16 & 1) * 8;                           // byte offset inside the granule

    float m_run[NQ], l_run[NQ];
    f32x16 o_acc[NQ][NDB];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_run[nq] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[nq][db][r] = 0.f;
    }

    const float c = p.scale_log2e;       // scale * log2(e), >= 0

    load_tile(0);
    store_tile(0);
    // Pin the Q fragments as "arrived" here: otherwise the loads stay pending into the loop and the
    // in-order memory counter makes the first MFMAs of every iteration wait for the K/V prefetch too.
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+v"(qf[nq][kk]));
    __syncthreads();

    for (int t = 0; t < nt; ++t) {
        const int buf = t & 1;
        if (t + 1 < nt) load_tile(t + 1);

        // ---- S^T = K Q^T
        f32x16 s[NQ][NKB];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[nq][kb][r] = 0.f;

        const unsigned char* kb_base = k_lds + buf * TILE_BYTES + k_row_off;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const int gsw = ((2 * kk + lh) ^ (li & (G - 1))) * 16;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb_base + kb * 32 * (D * 2) + gsw);
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq)
                    s[nq][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nq][kk], s[nq][kb], 0, 0, 0);
            }
        }

        // ---- key-padding tail: only the last tile can hold hidden keys
        const bool tail = (t + 1) * BN > n_v;
        if (tail) {
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = t * BN + kb * 32 + (r >> 2) * 8 + 4 * lh + (r & 3);
                    if (key >= n_v) {
#pragma unroll
                        for (int nq = 0; nq < NQ; ++nq) s[nq][kb][r] = -INFINITY;
                    }
                }
        }

        // ---- online softmax (fp32), probabilities packed to bf16 operands
        unsigned pfrag[NQ][NKB][2][4];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            float mx = s[nq][0][0];
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[nq][kb][r]);
            mx = pair_max(mx);
            const float m_new = fmaxf(m_run[nq], mx);
            if (__builtin_amdgcn_ballot_w64(m_new > m_run[nq]) != 0) {      // wave-uniform: rare after the first tiles
                // first tile: nothing accumulated yet (and -inf * 0 would be NaN for scale 0)
                const float alpha = m_run[nq] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_run[nq] - m_new) * c);
                l_run[nq] *= alpha;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[nq][db][r] *= alpha;
                m_run[nq] = m_new;
            }
            const float mc = m_run[nq] * c;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    s[nq][kb][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][kb][r], c, -mc));
            if (tail) {      // hidden keys get probability exactly 0 whatever the scale
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = t * BN + kb * 32 + (r >> 2) * 8 + 4 * lh + (r & 3);
                        if (key >= n_v) s[nq][kb][r] = 0.f;
                    }
            }
            float lsum = 0.f;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) lsum += s[nq][kb][r];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        pfrag[nq][kb][u][j] = pack_bf16(s[nq][kb][8 * u + 2 * j], s[nq][kb][8 * u + 2 * j + 1]);
            }
            l_run[nq] += lsum;
        }

        // ---- O^T += V^T P^T
        const unsigned char* vb_base = v_lds + buf * TILE_BYTES;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int key0 = kb * 32 + u * 16 + v_key_in;         // first 4-key read; second is +8
                // key0 % 4 == (t16>>2) % 4 and (key0+8) % 4 the same
                const int rsw = ((key0 & 3) << 2) & (G - 1);
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const int g = (db * 4 + v_colg) ^ rsw;
                    const int off0 = key0 * (D * 2) + g * 16 + v_sub;
                    const int off1 = off0 + 8 * (D * 2);
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(vb_base + off0));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(vb_base + off1));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq) {
                        u32x4 pv = {pfrag[nq][kb][u][0], pfrag[nq][kb][u][1], pfrag[nq][kb][u][2], pfrag[nq][kb][u][3]};
                        o_acc[nq][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pv),
                                                                                 o_acc[nq][db], 0, 0, 0);
                    }
                }
            }

        if (t + 1 < nt) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, write out and lse
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float l_tot = pair_sum(l_run[nq]);
        const float inv = 1.0f / l_tot;
        const int64_t row = q_row0 + nq * 32 + li;
        if (row < Sq) {
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 o4 = {o_acc[nq][db][4 * a] * inv, o_acc[nq][db][4 * a + 1] * inv,
                                o_acc[nq][db][4 * a + 2] * inv, o_acc[nq][db][4 * a + 3] * inv};
                    *reinterpret_cast<f32x4*>(op + row * D + db * 32 + a * 8 + 4 * lh) = o4;
                }
            if (lh == 0) lp[row] = m_run[nq] * p.scale + __logf(l_tot);
        }
    }
}

// out = 0, lse = -inf: the result of attention over an empty key set.
__global__ void attn_empty_kernel(const AttnParams p, int D) {
    const int bh = blockIdx.y;
    const int b = bh / p.Hg, h = bh - b * p.Hg;
    float* op = p.out + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs;
    __bf16* oph = reinterpret_cast<__bf16*>(p.out) + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs;
    float* lp = p.lse + (int64_t)b * p.l_bs + (int64_t)h * p.l_hs;
    const int64_t n = p.Sq * D;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        if (p.out_bf16) oph[i] = (__bf16)0.f;
        else op[i] = 0.f;
        if (i < p.Sq) lp[i] = -INFINITY;
    }
}

template <int D, int NQ, int NW, int BN, int MINB>
static hipError_t launch_variant(const AttnParams& p, int BH, hipStream_t st) {
    constexpr int M = 32 * NQ * NW;
    constexpr int smem = 4 * BN * D * 2;
    auto kern = attn_fwd_kernel<D, NQ, NW, BN, MINB>;
    static KernelSetup setup;
    hipError_t e = setup.ensure(reinterpret_cast<const void*>(kern), smem, nullptr);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((p.Sq + M - 1) / M), (unsigned)BH);
    hipLaunchKernelGGL(kern, grid, dim3(64 * NW), smem, st, p);
    return hipGetLastError();
}

hipError_t launch_attn_fwd(const AttnParams& p, int BH, int D, int variant, float* ws, int64_t ws_slots, hipStream_t st) {
    if (p.n_v == 0) {
        dim3 grid((unsigned)((p.Sq * D + 255) / 256 < 4096 ? (p.Sq * D + 255) / 256 : 4096), (unsigned)BH);
        hipLaunchKernelGGL(attn_empty_kernel, grid, dim3(256), 0, st, p, D);
        return hipGetLastError();
    }
    if (p.out_bf16 && variant != 3) variant = 0;                       // only the software-pipelined kernel writes bf16
    switch (variant) {
        case 1:                                                        // reference tiling, M=128, two workgroups per CU
            return D == 64 ? launch_variant<64, 1, 4, 64, 2>(p, BH, st) : launch_variant<128, 1, 4, 64, 2>(p, BH, st);
        case 2:                                                        // reference tiling, M=256, two waves per SIMD
            return D == 64 ? launch_variant<64, 1, 8, 64, 1>(p, BH, st) : launch_variant<128, 1, 8, 64, 1>(p, BH, st);
        case 3: {                                                      // software-pipelined kernel, second sweep forced
            AttnParams r = p;
            r.redo_always = 1;
            return launch_attn_fwd_sp(r, BH, D, ws, ws_slots, st);
        }
        default: return launch_attn_fwd_sp(p, BH, D, ws, ws_slots, st);              // software-pipelined kernel
    }
}

}  // namespace pda
