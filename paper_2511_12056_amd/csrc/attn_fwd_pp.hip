// Flash-attention forward, "ping-pong" schedule for gfx950 (d = 128): same tiling and MFMA
// formulation as attn_fwd.hip (S^T = K Q^T, O^T = V^T P^T on v_mfma_f32_32x32x16_bf16, one query
// per lane), with the matrix-core work and the softmax arithmetic of different wavefronts made to
// overlap by construction.
//
// A workgroup has 8 wavefronts = 2 per SIMD; wavefronts 0-3 form group A, 4-7 group B, and the
// two wavefronts that share a SIMD are in different groups.  Time is cut into phases closed by a
// workgroup barrier.  In every phase one group runs an MFMA block (PV of its previous key tile,
// then QK of its current one: 32 MFMAs) while the other runs a VALU block (the online softmax of
// its current tile: max, exp2, sum, bf16 packing), and the roles swap at the barrier.  B runs one
// phase behind A.  Both blocks take about the same time (1024 matrix-pipe cycles against ~950
// VALU cycles), so the matrix pipe of each SIMD always has a wavefront feeding it.
//
// K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4, no VGPR staging),
// three buffers per tensor.  At the start of its MFMA block t a wavefront issues its share of
// K tile t+2 and V tile t+1; they are first read four phases (A) or three phases (B) later, and
// the buffers they overwrite (K tile t-1, V tile t-2) were last read one phase earlier.  Before
// the barrier that closes every odd phase each wavefront waits for all but its latest batch.
// The LDS image of a tile is the swizzled layout described in attn_fwd.hip; since the DMA writes
// lane l's 16 bytes at position l of a 1 KB chunk, the swizzle is applied to the global address
// each lane fetches.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds_base + 16*l
// (lds_base wave-uniform, passed in M0).  Written as inline assembly on purpose: the compiler's
// wait-count insertion then does not see an LDS write it cannot disambiguate from the operand
// reads that follow (it would drain the whole prefetch before every LDS read); completion is
// tracked by hand with s_waitcnt vmcnt before the barriers.
__device__ __forceinline__ void lds_dma16(const void* gsrc, const void* lds_dst) {
    const unsigned lds_addr = (unsigned)(uintptr_t)(LDS_PTR(const void))lds_dst;
    unsigned saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"(lds_addr), "v"(gsrc)
                 : "memory");
}

template <int D, int PRIO>
__global__ __launch_bounds__(512, 1) void attn_fwd_pp_kernel(const AttnParams p) {
    constexpr int NW = 8;
    constexpr int BN = 64;
    constexpr int M = 32 * NW;            // 256 query rows per workgroup
    constexpr int G = D / 8;              // 16-byte granules per row
    constexpr int NKB = BN / 32;
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    constexpr int TILE_BYTES = BN * D * 2;
    constexpr int NBUF = 3;
    constexpr int CHUNKS = TILE_BYTES / 1024;      // 1 KB DMA chunks per tile
    constexpr int CPW = CHUNKS / NW;               // chunks per wavefront per tile
    constexpr int RPC = 1024 / (D * 2);            // rows per chunk
    static_assert(CHUNKS % NW == 0, "tile chunks must divide over the wavefronts");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* const k_lds = smem;                          // [3][BN][D] bf16
    unsigned char* const v_lds = smem + NBUF * TILE_BYTES;      // [3][BN][D] bf16

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const bool grp_b = wave >= 4;

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

    // ---- tile DMA: this wavefront's chunks; lane -> (row in tile, granule to fetch)
    int ld_row[CPW], ld_colk[CPW], ld_colv[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        const int cidx = wave * CPW + j;
        const int r = cidx * RPC + lane / G;
        const int gp = lane % G;                               // granule position the lane writes in LDS
        ld_row[j] = r;
        ld_colk[j] = (gp ^ (r & (G - 1))) * 8;                 // element offset of the granule it must fetch
        ld_colv[j] = (gp ^ (((r & 3) << 2) & (G - 1))) * 8;
    }
    auto issue_k = [&](int tile, int buf) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            int row = tile * BN + ld_row[j];
            row = row < n_v ? row : n_v - 1;                   // hidden / out-of-range keys are never read
            const __bf16* src = kp + (int64_t)row * D + ld_colk[j];
            unsigned char* dst = k_lds + buf * TILE_BYTES + (wave * CPW + j) * 1024;
            lds_dma16(src, dst);
        }
    };
    auto issue_v = [&](int tile, int buf) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            int row = tile * BN + ld_row[j];
            row = row < n_v ? row : n_v - 1;
            const __bf16* src = vp + (int64_t)row * D + ld_colv[j];
            unsigned char* dst = v_lds + buf * TILE_BYTES + (wave * CPW + j) * 1024;
            lds_dma16(src, dst);
        }
    };

    // prologue batch: K0, V0, K1
    issue_k(0, 0);
    issue_v(0, 0);
    issue_k(1, 1);

    // ---- Q operand fragments, resident for the whole sweep
    bf16x8 qf[NKK];
    {
        int64_t row = q_row0 + li;
        row = row < Sq ? row : Sq - 1;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            qf[kk] = *reinterpret_cast<const bf16x8*>(qp + row * D + kk * 16 + 8 * lh);
    }

    // ---- per-lane LDS read offsets (see attn_fwd.hip)
    const int k_row_off = li * (D * 2);
    const int t16 = lane & 15;
    const int v_key_in = 4 * lh + (t16 >> 2);
    const int v_colg = 2 * (li >> 4) + ((t16 & 3) >> 1);
    const int v_sub = (t16 & 1) * 8;

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o_acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
    f32x16 s[NKB];
    unsigned pfrag[NKB][2][4];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) pfrag[kb][u][j] = 0u;

    const float c = p.scale_log2e;

    // Steady-state MFMA block: PV of the previous tile then QK of the current one as one
    // straight-line region, with the LDS operand reads issued PF matrix instructions ahead of their
    // use (the scheduling directives below pin that interleaving), so that the matrix pipe does
    // not wait for LDS latency after the first few instructions.
    auto fused_block = [&](int vbuf, int kbuf_) {
        constexpr int PF = 4;
        const unsigned char* vb_base = v_lds + vbuf * TILE_BYTES;
        const unsigned char* kb_base = k_lds + kbuf_ * TILE_BYTES + k_row_off;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int key0 = kb * 32 + u * 16 + v_key_in;
                const int rsw = ((key0 & 3) << 2) & (G - 1);
                const u32x4 pv = {pfrag[kb][u][0], pfrag[kb][u][1], pfrag[kb][u][2], pfrag[kb][u][3]};
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const int g = (db * 4 + v_colg) ^ rsw;
                    const int off0 = key0 * (D * 2) + g * 16 + v_sub;
                    const int off1 = off0 + 8 * (D * 2);
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(vb_base + off0));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(vb_base + off1));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                        __builtin_bit_cast(bf16x8, pv), o_acc[db], 0, 0, 0);
                }
            }
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const int gsw = ((2 * kk + lh) ^ (li & (G - 1))) * 16;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(kb_base + kb * 32 * (D * 2) + gsw);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[kb], 0, 0, 0);
            }
        }
        // Issue order: reads for the first PF PV MFMAs, then one MFMA + the reads of the MFMA PF ahead.
        constexpr int N_PV = NKB * 2 * NDB, N_QK = NKK * NKB;
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * PF, 0);
#pragma unroll
        for (int i = 0; i < N_PV + N_QK; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            const int ahead = i + PF;
            if (ahead < N_PV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            else if (ahead < N_PV + N_QK) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    auto softmax_block = [&](int t) {
        const bool tail = (t + 1) * BN > n_v;
        if (tail) {
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = t * BN + kb * 32 + (r >> 2) * 8 + 4 * lh + (r & 3);
                    if (key >= n_v) s[kb][r] = -INFINITY;
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
        mx = pair_max(mx);
        const float m_new = fmaxf(m_run, mx);
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {          // wave-uniform, rare after the first tiles
            const float alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_run - m_new) * c);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
            m_run = m_new;
        }
        const float mc = m_run * c;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], c, -mc));
        if (tail) {              // hidden keys get probability exactly 0 whatever the scale
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = t * BN + kb * 32 + (r >> 2) * 8 + 4 * lh + (r & 3);
                    if (key >= n_v) s[kb][r] = 0.f;
                }
        }
        float lsum = 0.f;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) lsum += s[kb][r];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j) pfrag[kb][u][j] = pack_bf16(s[kb][8 * u + 2 * j], s[kb][8 * u + 2 * j + 1]);
        }
        l_run += lsum;
    };

    // All but the newest batch (CPW K chunks + CPW V chunks) of this wavefront's DMA have landed.
    auto wait_older_batches = [&]() {
        if constexpr (2 * CPW == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
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
    if (grp_b) barrier();                    // B runs one phase behind A

    // Iteration t of a wavefront: MFMA block [PV(t-1), QK(t)], barrier, VALU block softmax(t),
    // barrier.  t runs to nt inclusive so that the last PV has a block of its own.
    int kbuf = 0;                            // buffer index of K tile t and of V tile t
    int vprev = NBUF - 1;                    // buffer index of V tile t-1
    for (int t = 0; t <= nt; ++t) {
        const int nxt = kbuf == NBUF - 1 ? 0 : kbuf + 1;   // (t+1) % 3
        issue_k(t + 2, vprev);                              // (t+2) % 3 == (t-1) % 3
        issue_v(t + 1, nxt);
        if (PRIO == 1) __builtin_amdgcn_s_setprio(1);
        // Same block every iteration: at t = 0 the probabilities are still zero (PV adds nothing,
        // read from the already loaded V tile 0), at t = nt the scores of the clamped tile are unused.
        fused_block(t > 0 ? vprev : 0, kbuf);
        if (PRIO == 1) __builtin_amdgcn_s_setprio(0);
        if (grp_b) wait_older_batches();
        barrier();
        if (PRIO == 2) __builtin_amdgcn_s_setprio(1);
        if (t < nt) softmax_block(t);
        if (PRIO == 2) __builtin_amdgcn_s_setprio(0);
        if (!grp_b) wait_older_batches();
        barrier();
        vprev = kbuf;
        kbuf = nxt;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // no DMA may outlive the workgroup's LDS
    if (!grp_b) barrier();                                  // even out the barrier count with B's extra one

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

template <int PRIO>
static hipError_t launch_pp(const AttnParams& p, int BH, hipStream_t st) {
    constexpr int D = 128;
    constexpr int smem = 2 * 3 * 64 * D * 2;
    auto kern = attn_fwd_pp_kernel<D, PRIO>;
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

hipError_t launch_attn_fwd_pp(const AttnParams& p, int BH, int mode, hipStream_t st) {
    switch (mode) {
        case 1:  return launch_pp<1>(p, BH, st);
        case 2:  return launch_pp<2>(p, BH, st);
        default: return launch_pp<0>(p, BH, st);
    }
}

}  // namespace pda
