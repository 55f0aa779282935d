// Flash-attention forward, software-pipelined ("interleaved") schedule for gfx950, d = 128.
//
// Same tiling and MFMA formulation as attn_fwd.hip (S^T = K Q^T, O^T = V^T P^T on
// v_mfma_f32_32x32x16_bf16, one query per lane, 8 wavefronts x 32 query rows per workgroup,
// 64-key tiles).  What differs is when things run.  On this hardware the matrix pipe is fed
// through the VALU issue port: an MFMA holds the port for 8 of its 32 cycles, an ordinary VALU op
// for 4, a transcendental for 8.  The softmax of one tile costs about as much port time as the
// tile's MFMAs cost matrix-pipe time, so the two must overlap at instruction granularity.  Each
// wavefront therefore runs ONE instruction stream per key tile t in which three independent
// pieces of work are interleaved:
//
//     matrix pipe:   PV(t-1)  (O += V_{t-1} P_{t-1})   then   QK(t+1)  (S_{t+1} = K_{t+1} Q^T)
//     VALU:          softmax(t):  S_t -> running max / sum, P_t (bf16)
//     LDS reads:     operands of the MFMAs, issued PF instructions ahead of their use
//
// The issue order is pinned with scheduling directives (one MFMA, its look-ahead LDS reads, a few
// VALU ops, repeat).  Two wavefronts share a SIMD and run the same mixed stream, so whenever one
// waits the other issues.  The O accumulators are rescaled after the stream (PV(t-1) must land
// before the factor of tile t is applied), and only when the running max of some lane moved by
// more than 2^8: otherwise the old reference is kept, which is exact because the final
// normalisation uses the same reference.
//
// K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4), three buffers per
// tensor: at the top of iteration t a wavefront issues its share of K tile t+3 and V tile t+1
// (both buffers were last read in iteration t-1); they are first read in iteration t+2.  Before
// the single barrier that closes an iteration each wavefront waits for all but its newest batch.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

// 16 bytes per lane from global memory (scalar base + per-lane byte offset) straight into LDS:
// lane l's data lands at lds_base + 16*l (lds_base wave-uniform, passed in M0).  Inline assembly
// on purpose: the compiler's wait-count insertion then does not see an LDS write that it cannot
// tell apart from the operand reads that follow (it would drain the whole prefetch before every
// LDS read); completion is tracked by hand with s_waitcnt vmcnt before the barrier.
__device__ __forceinline__ void lds_dma16_s(const void* sbase, unsigned voff, const void* lds_dst) {
    const unsigned lds_addr = (unsigned)(uintptr_t)(LDS_PTR(const void))lds_dst;
    unsigned saved_m0;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
        : "=&s"(saved_m0)
        : "s"(lds_addr), "v"(voff), "s"(sbase)
        : "memory");
}

template <int D>
__global__ __launch_bounds__(512, 1) void attn_fwd_il_kernel(const AttnParams p) {
    constexpr int NW = 8;
    constexpr int BN = 64;
    constexpr int M = 32 * NW;
    constexpr int G = D / 8;
    constexpr int NKB = BN / 32;
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    constexpr int TILE_BYTES = BN * D * 2;
    constexpr int NBUF = 3;
    constexpr int CHUNKS = TILE_BYTES / 1024;
    constexpr int CPW = CHUNKS / NW;
    constexpr int RPC = 1024 / (D * 2);
    static_assert(CHUNKS % NW == 0 && CPW == 2, "DMA batch size is fixed below");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* const k_lds = smem;                          // [3][BN][D] bf16
    unsigned char* const v_lds = smem + NBUF * TILE_BYTES;      // [3][BN][D] bf16

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;

    const int bh = blockIdx.y;
    const int b = bh / p.Hg, h = bh - b * p.Hg;
    const __bf16* __restrict__ qp = p.q + (int64_t)b * p.q_bs + (int64_t)h * p.q_hs;
    const __bf16* __restrict__ kp = p.k + (int64_t)b * p.kv_bs + (int64_t)h * p.kv_hs;
    const __bf16* __restrict__ vp = p.v + (int64_t)b * p.kv_bs + (int64_t)h * p.kv_hs;
    float* __restrict__ op = p.out + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs;
    float* __restrict__ lp = p.lse + (int64_t)b * p.l_bs + (int64_t)h * p.l_hs;

    const int64_t Sq = p.Sq;
    const int n_v = (int)p.n_v;                       // >= 1
    const int nt = (n_v + BN - 1) / BN;
    const int64_t q_row0 = (int64_t)blockIdx.x * M + wave * 32;

    // ---- tile DMA: this wavefront's two 1 KB chunks of a tile; lane -> (row, granule to fetch)
    int ld_row[CPW];
    unsigned ld_offk[CPW], ld_offv[CPW];              // byte offset inside the tile of the granule to fetch
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        const int cidx = wave * CPW + j;
        const int r = cidx * RPC + lane / G;
        const int gp = lane % G;                      // granule position the lane's data lands on
        ld_row[j] = r;
        ld_offk[j] = (unsigned)(r * D * 2 + (gp ^ (r & (G - 1))) * 16);
        ld_offv[j] = (unsigned)(r * D * 2 + (gp ^ (((r & 3) << 2) & (G - 1))) * 16);
    }
    auto issue_tile = [&](const __bf16* base, const unsigned (&offs)[CPW], unsigned char* lds_tile, int tile) {
        if ((tile + 1) * BN <= n_v) {                 // whole tile valid: scalar tile base + fixed lane offsets
            const __bf16* tbase = base + (int64_t)tile * BN * D;
#pragma unroll
            for (int j = 0; j < CPW; ++j) lds_dma16_s(tbase, offs[j], lds_tile + (wave * CPW + j) * 1024);
        } else {                                      // tail or beyond: rows clamped to the last valid key
            const int last_tile = (n_v - 1) / BN;
            const int tb = tile < last_tile ? tile : last_tile;
            const __bf16* tbase = base + (int64_t)tb * BN * D;
#pragma unroll
            for (int j = 0; j < CPW; ++j) {
                int row = tile * BN + ld_row[j];
                row = row < n_v ? row : n_v - 1;      // hidden / out-of-range keys are never read
                const unsigned off = (unsigned)(row - tb * BN) * (D * 2) + (offs[j] & (D * 2 - 1));
                lds_dma16_s(tbase, off, lds_tile + (wave * CPW + j) * 1024);
            }
        }
    };

    // prologue batch: K0, K1, K2, V0
    issue_tile(kp, ld_offk, k_lds + 0 * TILE_BYTES, 0);
    issue_tile(kp, ld_offk, k_lds + 1 * TILE_BYTES, 1);
    issue_tile(kp, ld_offk, k_lds + 2 * TILE_BYTES, 2);
    issue_tile(vp, ld_offv, v_lds + 0 * TILE_BYTES, 0);

    // ---- Q operand fragments, resident for the whole sweep
    bf16x8 qf[NKK];
    {
        int64_t row = q_row0 + li;
        row = row < Sq ? row : Sq - 1;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            qf[kk] = *reinterpret_cast<const bf16x8*>(qp + row * D + kk * 16 + 8 * lh);
    }

    // ---- per-lane LDS read offsets (layout: see attn_fwd.hip)
    const int k_row_off = li * (D * 2);
    const int t16 = lane & 15;
    const int v_key_in = 4 * lh + (t16 >> 2);
    const int v_colg = 2 * (li >> 4) + ((t16 & 3) >> 1);
    const int v_sub = (t16 & 1) * 8;

    float m_run = -INFINITY;         // reference max of the running sums (raw score units)
    float l_run = 0.f;               // this lane's share of the running sum
    f32x16 o_acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
    f32x16 s_a[NKB], s_b[NKB];       // scores of two consecutive tiles, alternating roles
    unsigned p_a[NKB][2][4], p_b[NKB][2][4];   // packed bf16 P of two consecutive tiles (MFMA operand order)
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) p_a[kb][u][j] = p_b[kb][u][j] = 0u;

    const float c = p.scale_log2e;   // > 0 (the host substitutes a tiny positive value for scale 0)

    auto mask_tail = [&](f32x16 (&s)[NKB], int t) {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = t * BN + kb * 32 + (r >> 2) * 8 + 4 * lh + (r & 3);
                if (key >= n_v) s[kb][r] = -INFINITY;
            }
    };

    auto barrier = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };

    // Q fragments and the prologue tiles have arrived
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+v"(qf[kk]));
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    barrier();

    // ---- S_0 = K_0 Q^T (not overlapped with anything)
    {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s_a[kb][r] = 0.f;
        const unsigned char* kb_base = k_lds + k_row_off;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const int gsw = ((2 * kk + lh) ^ (li & (G - 1))) * 16;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb_base + kb * 32 * (D * 2) + gsw);
                s_a[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s_a[kb], 0, 0, 0);
            }
        }
        if (BN > n_v) mask_tail(s_a, 0);
    }
    barrier();           // K tile 0 is overwritten by the first DMA of the loop

    int kn = 1;          // buffer of K tile t+1
    int vp_ = 0;         // buffer of V tile t-1 (tile 0's buffer at t = 0, where P is still zero)
    int vc = 0;          // buffer of V tile t
    // One iteration.  s_c: scores of tile t (in, overwritten by its probabilities); s_n: scores of
    // tile t+1 (out); p_in: packed P of tile t-1 (in); p_out: packed P of tile t (out).
    //
    // The body is written slot by slot in the order it is meant to issue, and a scheduling barrier
    // after every slot keeps the compiler from regrouping it.  Slot i (0..31) = MFMA i (PV 0..15,
    // then QK 0..15), the LDS reads of MFMA i+PF, and the i-th slice of the softmax VALU work:
    // slots 0-3 the row max, 4-5 the reference/rescale factors, 6-31 the 32 exponentials with
    // their packing to bf16 and the row sum.
    auto iteration = [&](int t, f32x16 (&s_c)[NKB], f32x16 (&s_n)[NKB], unsigned (&p_in)[NKB][2][4],
                         unsigned (&p_out)[NKB][2][4]) {
        // DMA: K tile t+3 replaces K tile t, V tile t+1 replaces V tile t-2
        {
            const int k3 = kn == 0 ? NBUF - 1 : kn - 1;               // (t+3) % 3 == t % 3
            const int v1 = vc == NBUF - 1 ? 0 : vc + 1;               // (t+1) % 3
            issue_tile(kp, ld_offk, k_lds + k3 * TILE_BYTES, t + 3);
            issue_tile(vp, ld_offv, v_lds + v1 * TILE_BYTES, t + 1);
        }

        constexpr int N_PV = NKB * 2 * NDB, N_QK = NKK * NKB, N_MM = N_PV + N_QK;
        constexpr int PF = 3, RING = 4;
        static_assert(N_MM == 32 && NKB == 2 && NDB == 4, "slot plan below is written for d = 128, 64-key tiles");
        bf16x8 frag[RING];
        const unsigned char* vb_base = v_lds + vp_ * TILE_BYTES;
        const unsigned char* kb_base = k_lds + kn * TILE_BYTES + k_row_off;

        auto load_frag = [&](auto idx) {
            constexpr int i = decltype(idx)::value;
            if constexpr (i < N_PV) {
                constexpr int kb = i / 8, u = (i / 4) % 2, db = i % 4;
                const int key0 = kb * 32 + u * 16 + v_key_in;
                const int rsw = ((key0 & 3) << 2) & (G - 1);
                const int g = (db * 4 + v_colg) ^ rsw;
                const int off0 = key0 * (D * 2) + g * 16 + v_sub;
                const int off1 = off0 + 8 * (D * 2);
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(vb_base + off0));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(vb_base + off1));
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                frag[i % RING] = __builtin_bit_cast(bf16x8, av);
            } else if constexpr (i < N_MM) {
                constexpr int j = i - N_PV, kk = j / 2, kb = j % 2;
                const int gsw = ((2 * kk + lh) ^ (li & (G - 1))) * 16;
                frag[i % RING] = *reinterpret_cast<const bf16x8*>(kb_base + kb * 32 * (D * 2) + gsw);
            }
        };
        auto do_mfma = [&](auto idx) {
            constexpr int i = decltype(idx)::value;
            if constexpr (i < N_PV) {
                constexpr int kb = i / 8, u = (i / 4) % 2, db = i % 4;
                const u32x4 pv = {p_in[kb][u][0], p_in[kb][u][1], p_in[kb][u][2], p_in[kb][u][3]};
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i % RING], __builtin_bit_cast(bf16x8, pv),
                                                                    o_acc[db], 0, 0, 0);
            } else {
                constexpr int j = i - N_PV, kk = j / 2, kb = j % 2;
                if constexpr (kk == 0) {
                    const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    s_n[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i % RING], qf[kk], zero, 0, 0, 0);
                } else {
                    s_n[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i % RING], qf[kk], s_n[kb], 0, 0, 0);
                }
            }
        };

        // softmax state of this tile
        float mx = s_c[0][0];
        float m_use = 0.f, alpha = 1.f, mc = 0.f, lsum = 0.f;
        auto pack_pair = [&](auto qidx) {       // pair q = elements 2q, 2q+1 of the 32 this lane holds
            constexpr int q = decltype(qidx)::value;
            constexpr int kb = q / 8, u = (q % 8) / 4, j = q % 4;
            const unsigned pk = pack_bf16(s_c[kb][8 * u + 2 * j], s_c[kb][8 * u + 2 * j + 1]);
            p_out[kb][u][j] = pk;
            // row sum over the ROUNDED probabilities, two per instruction (v_dot2c_f32_bf16)
            lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk),
                                                   __builtin_bit_cast(bf16x2, 0x3f803f80u), lsum, false);
        };
        auto valu_slice = [&](auto idx) {
            constexpr int i = decltype(idx)::value;
            if constexpr (i < 4) {                                  // row max over the lane's 32 scores
#pragma unroll
                for (int e = 8 * i; e < 8 * i + 8; e += 2)
                    mx = fmaxf(fmaxf(mx, s_c[e / 16][e % 16]), s_c[(e + 1) / 16][(e + 1) % 16]);
            } else if constexpr (i == 4) {
                mx = pair_max(mx);
                // keep the old reference unless the max moved by more than 2^8 (in exp2 units)
                const float m_new = fmaxf(m_run, mx);
                const bool move = (m_new - m_run) * c > 8.0f || m_run == -INFINITY;
                m_use = move ? m_new : m_run;
            } else if constexpr (i == 5) {
                alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_run - m_use) * c);
                mc = m_use * c;
            } else {                                                // 32 exponentials over 26 slots
                constexpr int k = i - 6;
                constexpr int h0 = k * 32 / 26, h1 = (k + 1) * 32 / 26;
                static_for<h0, h1>([&](auto hidx) {
                    constexpr int e = decltype(hidx)::value;
                    if constexpr (e % 2 == 0 && e >= 2) pack_pair(std::integral_constant<int, e / 2 - 1>{});
                    s_c[e / 16][e % 16] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_c[e / 16][e % 16], c, -mc));
                });
            }
        };

        // ================= interleaved region: softmax(t) | PV(t-1), QK(t+1) =================
        static_for<0, PF>([&](auto i) { load_frag(i); });
        static_for<0, N_MM>([&](auto idx) {
            constexpr int i = decltype(idx)::value;
            do_mfma(idx);
            load_frag(std::integral_constant<int, i + PF>{});
            valu_slice(idx);
            __builtin_amdgcn_sched_barrier(0);
        });
        pack_pair(std::integral_constant<int, 15>{});
        l_run = __builtin_fmaf(l_run, alpha, lsum);
        m_run = m_use;
        // =====================================================================================

        // rescale O once PV(t-1) is in, if some lane moved its reference (rare after the first tiles)
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
        }
        if ((t + 2) * BN > n_v) mask_tail(s_n, t + 1);     // S_{t+1} holds hidden keys

        // rotate the buffer indices: tile t+1 becomes current
        vp_ = vc;
        vc = vc == NBUF - 1 ? 0 : vc + 1;
        kn = kn == NBUF - 1 ? 0 : kn + 1;

        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");     // all but this iteration's batch have landed
        barrier();
    };

    // The loop runs over tiles 0 .. nt (the extra one only completes PV(nt-1): its scores are all
    // hidden, so its probabilities are zero), rounded up to an even count so that the score and
    // probability registers can alternate roles without copies.
    const int t_end = (nt + 2) & ~1;
    for (int t = 0; t < t_end; t += 2) {
        iteration(t, s_a, s_b, p_b, p_a);
        iteration(t + 1, s_b, s_a, p_a, p_b);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // no DMA may outlive the workgroup's LDS

    // ---- epilogue: normalise, write out and lse
    const float l_tot = pair_sum(l_run);
    const float inv = 1.0f / l_tot;
    const int64_t row = q_row0 + li;
    if (row < Sq) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 o4 = {o_acc[db][4 * a] * inv, o_acc[db][4 * a + 1] * inv, o_acc[db][4 * a + 2] * inv,
                            o_acc[db][4 * a + 3] * inv};
                *reinterpret_cast<f32x4*>(op + row * D + db * 32 + a * 8 + 4 * lh) = o4;
            }
        if (lh == 0) lp[row] = m_run * p.scale + __logf(l_tot);
    }
}

hipError_t launch_attn_fwd_il(const AttnParams& p, int BH, hipStream_t st) {
    constexpr int D = 128;
    constexpr int smem = 2 * 3 * 64 * D * 2;
    auto kern = attn_fwd_il_kernel<D>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)((p.Sq + 255) / 256), (unsigned)BH);
    hipLaunchKernelGGL(kern, grid, dim3(512), smem, st, p);
    return hipGetLastError();
}

}  // namespace pda
