// Flash-attention forward, software-pipelined schedule for gfx950, d = 128, 64-key tiles,
// 256 query rows per workgroup.  Template parameter NQ = number of 32-row query sub-tiles a
// wavefront owns.  Only NQ = 1 (8 wavefronts, two per SIMD) is instantiated.  NQ = 2 (one wavefront
// per SIMD, each K/V operand fragment feeding two MFMAs, half the LDS operand reads) needs the O
// accumulators and Q fragments in accumulation registers, which the compiler only does when the
// MFMAs are written in assembly; built that way it was slower (a single wavefront per SIMD leaves
// the latencies at the iteration boundary exposed).
//
// MFMA formulation and LDS tile layout are those of attn_fwd.hip (S^T = K Q^T, O^T = V^T P^T on
// v_mfma_f32_32x32x16_bf16, one query per lane, XOR-swizzled 16-byte granules).  Schedule: on
// this hardware the matrix pipe is fed through the VALU issue port (an MFMA holds it for 8 of its
// 32 cycles, a plain VALU op for ~4, a transcendental for ~8), and the softmax of a tile needs
// about as much port time as the tile's MFMAs need matrix-pipe time.  Each wavefront therefore
// runs one instruction stream per key tile t that interleaves three independent pieces of work:
//
//     matrix pipe:   PV(t-1)  (O += V_{t-1} P_{t-1})   then   QK(t+1)  (S_{t+1} = K_{t+1} Q^T)
//     VALU:          softmax(t):  S_t -> running max / sum, P_t (bf16)
//     LDS reads:     MFMA operand fragments, issued PF slots ahead of their use
//
// written slot by slot in issue order (a scheduling barrier after every slot keeps that order).
//
// Softmax reference.  The value of softmax does not depend on the reference that is subtracted
// before the exponential, only overflow and underflow do, and fp32 (and bf16, which shares its
// exponent range) leaves a wide margin.  The item is therefore first swept with a FIXED reference per
// row, the max of the row's scores in the first key tile: no max pass, no rescaling of O, weights
// may exceed 1.  If a row's sum ends up beyond 2^64 (some later score lay that far above the
// first tile, or the input held non-finite values), or an output accumulator is not finite (large
// weights times large V entries), the workgroup sweeps the item again with the
// usual running max, where the reference moves only when the max grew by more than 2^8 and O is
// rescaled after the stream in a rare wave-uniform branch.  The row sum is taken with plain fp32
// adds on the unrounded probabilities; the dot-product instructions (v_dot2c_f32_bf16), which
// would sum two rounded ones at a time, occupy the matrix pipe and stall the MFMA stream.
//
// K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4), four buffers per
// tensor; the loop is unrolled four times so that every buffer offset is an immediate.  At the
// top of iteration t a wavefront issues its share of K tile t+4 (over K tile t) and V tile t+2
// (over V tile t-2), both last read in iteration t-1; before the barrier that closes the
// iteration it waits for all but its two newest batches, i.e. for K tile t+2 and V tile t, which
// iteration t+1 reads.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_internal.h"
#include "attn_device.h"

namespace pda {

// 16 bytes per lane from global memory (scalar base + per-lane byte offset) straight into LDS:
// lane l's data lands at lds_addr + 16*l (lds_addr wave-uniform, passed in M0).  Inline assembly
// on purpose: the compiler's wait-count insertion then does not see an LDS write that it cannot
// tell apart from the operand reads that follow (it would drain the whole prefetch before every
// LDS read); completion is tracked by hand with s_waitcnt vmcnt before the barrier.
// M0 is not restored; it is declared clobbered.
__device__ __forceinline__ void lds_dma16(const void* sbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// Same with the LDS address given as wave-uniform base + compile-time offset.
template <int LDS_OFF>
__device__ __forceinline__ void lds_dma16_at(const void* sbase, unsigned voff, unsigned lds_base) {
    asm volatile("s_add_u32 m0, %0, %1\n\tglobal_load_lds_dwordx4 %2, %3"
                 :
                 : "s"(lds_base), "n"(LDS_OFF), "v"(voff), "s"(sbase)
                 : "memory", "scc", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N == 4 || N == 8 || N == 16 || N == 0, "add the literal below");
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
}

// BASE2: the scores are already in units of log2 (the caller folded scale*log2(e) into Q), so the
// weights are 2^(q.k) and the first sweep needs no arithmetic before the exponential at all: the
// score accumulators start from minus the row's reference instead of from zero.
// Row-dependent XOR applied to the index of a row's 16-byte granules in an LDS tile, chosen so that
// the operand reads are free of bank conflicts (64 banks of 4 bytes).  With 256-byte rows (d = 128)
// every row starts at bank 0: the K reads (16 rows, one granule each) need 16 different granules,
// the transposing V reads (4 rows, 4 granules each) 4 different groups of 4.  With 128-byte rows
// (d = 64) even and odd rows already lie in different halves of the banks, so the XOR is taken
// from the row index without its lowest bit.
template <int D>
__device__ __forceinline__ constexpr int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D>
__device__ __forceinline__ constexpr int swz_v(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }

template <int D, int NQ, bool BASE2>
__global__ __launch_bounds__(512 / NQ, 1) void attn_fwd_sp_kernel(const AttnParams p) {
    static_assert(D == 128 || D == 64, "head dimension");
    constexpr int NW = 8 / NQ;            // wavefronts
    constexpr int BN = 64;
    constexpr int M = 256;
    constexpr int G = D / 8;              // 16-byte granules per row: 16 (d = 128) or 8
    constexpr int NKB = BN / 32;          // 2
    constexpr int NKK = D / 16;           // 8 or 4
    constexpr int NDB = D / 32;           // 4 or 2
    constexpr int TILE = BN * D * 2;      // 16 KB or 8 KB
    constexpr int NBUF = 4;
    constexpr int K_BASE = 0, V_BASE = NBUF * TILE;       // LDS byte offsets
    constexpr int CHUNKS = TILE / 1024;   // DMA chunks of 1 KB per tile: 16 or 8
    constexpr int CPW = CHUNKS / NW;      // per wavefront: 2 (4 with NQ = 2), or 1 for d = 64
    constexpr int RPC = 1024 / (D * 2);   // rows per chunk: 4 or 8
    static_assert(CPW >= 1, "every wavefront fetches at least one chunk of a tile");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int next_item;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;

    // Persistent workgroups (one per CU) take work items in index order from a device counter: the
    // chip's XCDs run at persistently different speeds (several percent apart under the power
    // limit) and the hardware deals the workgroups of a grid to them round robin, so a grid with
    // one workgroup per item would end with the slowest XCD while the others idle.  A launch with no
    // more items than workgroups needs no counter: workgroup i takes item i and leaves.
    const bool direct = p.n_items <= (int)gridDim.x;
    for (int round = 0;; ++round) {
    int item;
    if (direct) {
        item = round == 0 ? (int)blockIdx.x : p.n_items;
    } else {
        if (tid == 0) next_item = atomicAdd(p.counter, 1);
        __syncthreads();
        item = __builtin_amdgcn_readfirstlane(next_item);
        __syncthreads();                               // everyone has read it before the next fetch overwrites it
    }
    if (item >= p.n_items) break;

    // ---- work item -> (query tile, head, key range).  Items [0, n_full) are whole tiles; then the
    // cut tiles' key ranges, range-major, so that the items in flight at any time sweep the same keys.
    int tile = item, part = 0;
    if (item >= p.n_full) {
        const int idx = item - p.n_full;
        part = idx / p.n_cut;
        tile = p.n_full + (idx - part * p.n_cut);
    }
    const int bh = tile / p.tiles_per_head;
    const int q_tile = tile - bh * p.tiles_per_head;
    const int b = bh / p.Hg, h = bh - b * p.Hg;
    // this item's key range [kv0, kv1) (tile aligned): all keys, or range `part` of a cut tile
    int64_t kv0 = 0, kv1 = p.n_v;
    if (p.split > 1 && tile >= p.n_full) {
        kv0 = p.part_off[part];
        kv1 = p.part_off[part + 1];
    }
    const __bf16* __restrict__ qp = p.q + (int64_t)b * p.q_bs + (int64_t)h * p.q_hs;
    const __bf16* __restrict__ kp = p.k + (int64_t)b * p.kv_bs + (int64_t)h * p.kv_hs + kv0 * D;
    const __bf16* __restrict__ vp = p.v + (int64_t)b * p.kv_bs + (int64_t)h * p.kv_hs + kv0 * D;
    // part 0 writes the tile's rows of out/lse; later parts write rows 0..255 of their partial slot
    float* __restrict__ op;
    float* __restrict__ lp;
    int64_t row_sub;                                   // subtracted from the global row on store
    // With a bf16 `out` the merge pass needs fp32 partials of ALL parts of a cut tile, part 0 included.
    const bool cut = p.split > 1 && tile >= p.n_full;
    const bool to_ws = part > 0 || (cut && p.out_bf16);
    if (!to_ws) {
        op = p.out + (p.out_bf16 ? 0 : (int64_t)b * p.o_bs + (int64_t)h * p.o_hs);
        lp = p.lse + (int64_t)b * p.l_bs + (int64_t)h * p.l_hs;
        row_sub = 0;
    } else {
        const int64_t slot = p.out_bf16 ? (int64_t)(tile - p.n_full) * p.split + part
                                        : (int64_t)(tile - p.n_full) * (p.split - 1) + (part - 1);
        op = p.part_out + slot * (M * D);
        lp = p.part_lse + slot * M;
        row_sub = (int64_t)q_tile * M;
    }
    __bf16* __restrict__ oph = reinterpret_cast<__bf16*>(p.out) + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs;
    const bool store_bf16 = p.out_bf16 && !to_ws;

    const int64_t Sq = p.Sq;
    const int n_v = (int)(kv1 - kv0);                 // keys of this item, >= 1
    const int nt = (n_v + BN - 1) / BN;
    const int64_t q_row0 = (int64_t)q_tile * M + wave * (32 * NQ);
    const unsigned lds0 = (unsigned)(uintptr_t)(LDS_PTR(const void))smem;

    // ---- tile DMA: wavefront w fetches the 1 KB chunks w, w+NW, ... of a tile (4 key rows each).
    // Lane -> (row, granule to fetch); with this assignment row % 32 does not depend on the chunk
    // number, so one per-lane offset serves all of a wavefront's chunks.
    const int ld_row0 = wave * RPC + lane / G;        // row of chunk 0; chunk j adds j*NW*RPC
    const int ld_gp = lane % G;                       // granule position the lane's data lands on
    const unsigned ld_offk = (unsigned)(ld_row0 * D * 2 + (ld_gp ^ swz_k<D>(ld_row0)) * 16);
    const unsigned ld_offv = (unsigned)(ld_row0 * D * 2 + (ld_gp ^ swz_v<D>(ld_row0)) * 16);
    // chunk j (0..CPW-1) of this wavefront's share of a tile
    auto issue_chunk = [&](const __bf16* base, unsigned off0, unsigned lds_tile, int tile, int j) {
        const unsigned dst = lds0 + lds_tile + wave * 1024 + j * (NW * 1024);
        if ((tile + 1) * BN <= n_v) {                 // whole tile valid: scalar tile base + fixed lane offsets
            lds_dma16(base + (int64_t)tile * BN * D, off0 + j * (NW * 1024), dst);
        } else {                                      // tail or beyond: rows clamped to the last valid key
            const int last_tile = (n_v - 1) / BN;
            const int tb = tile < last_tile ? tile : last_tile;
            int row = tile * BN + ld_row0 + j * (NW * RPC);
            row = row < n_v ? row : n_v - 1;          // hidden / out-of-range keys are never read
            const unsigned off = (unsigned)(row - tb * BN) * (D * 2) + (off0 & (D * 2 - 1));
            lds_dma16(base + (int64_t)tb * BN * D, off, dst);
        }
    };
    const unsigned dma_base = lds0 + wave * 1024;
    unsigned ld_k[CPW], ld_v[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        ld_k[j] = ld_offk + j * (NW * 1024);
        ld_v[j] = ld_offv + j * (NW * 1024);
    }
    const __bf16* k_dma = kp + 4 * BN * D;            // K tile t+4 and V tile t+2 of the coming iteration
    const __bf16* v_dma = vp + 2 * BN * D;
    auto issue_tile = [&](const __bf16* base, unsigned off0, unsigned lds_tile, int tile) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) issue_chunk(base, off0, lds_tile, tile, j);
    };

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

    // ---- per-lane LDS operand addresses (loop invariant; buffer and block offsets are immediates)
    // K operand: row kb*32+li, granule (2kk+lh) ^ swz_k(li)
    LDS_PTR(const unsigned char) k_ptr[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) k_ptr[kk] = (LDS_PTR(const unsigned char))smem + (K_BASE + li * (D * 2) + (((2 * kk + lh) ^ swz_k<D>(li)) * 16));
    // V^T operand through the transposing read: within a 16-lane block, lane t supplies the address
    // of 4 consecutive columns (t%4) of key row (t/4) and receives column t of those 4 rows.
    const int t16 = lane & 15;
    const int v_key_in = 4 * lh + (t16 >> 2);                  // key inside a 16-key group (first 4-key read)
    LDS_PTR(const unsigned char) v_ptr[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
        const int g = (db * 4 + 2 * (li >> 4) + ((t16 & 3) >> 1)) ^ swz_v<D>(v_key_in);
        v_ptr[db] = (LDS_PTR(const unsigned char))smem + (V_BASE + v_key_in * (D * 2) + g * 16 + (t16 & 1) * 8);
    }

    float mc_run[NQ], l_run[NQ];     // reference max in exp2 units (max * scale * log2 e), lane's share of the running sum
    f32x16 o_acc[NQ][NDB];
    f32x16 nref[NQ];                                   // BASE2, first sweep: minus the row's reference, as an accumulator seed
    f32x16 s_a[NQ][NKB], s_b[NQ][NKB];                 // scores of two consecutive tiles, alternating roles
    // Packed bf16 P (MFMA operand order).  One buffer serves two consecutive tiles: group (kb,u) of
    // tile t-1 is consumed by the PV MFMAs of slots (d/32)(2kb+u) .. +d/32-1, before the softmax of tile t writes it.
    unsigned p_io[NQ][NKB][2][4];
    const float c = BASE2 ? 1.0f : p.scale_log2e;   // > 0 (the host substitutes a tiny positive value for scale 0)

    auto mask_tail = [&](f32x16 (&s)[NQ][NKB], int t) {
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
    };
    auto barrier = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };

    // One sweep over the item's keys.  SAFE = false (first attempt): the reference of a row is the
    // max of its scores in the first key tile and never moves, so the loop carries no max pass and
    // no rescaling; probabilities may exceed 1.  That is exact as long as nothing overflows, which
    // the caller of the sweep checks on the row sums.  SAFE = true: running max with lazy updates.
    auto sweep = [&](auto safe_c) {
        constexpr bool SAFE = decltype(safe_c)::value;
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            mc_run[nq] = -INFINITY;
            l_run[nq] = 0.f;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[nq][db][r] = 0.f;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) p_io[nq][kb][u][j] = 0u;
        }
        k_dma = kp + 4 * BN * D;
        v_dma = vp + 2 * BN * D;
        // prologue: K tiles 0..3, V tiles 0..1; V buffer 3 (read by the first, all-zero-weight PV) is zeroed
        issue_tile(kp, ld_offk, K_BASE + 0 * TILE, 0);
        issue_tile(vp, ld_offv, V_BASE + 0 * TILE, 0);
        issue_tile(kp, ld_offk, K_BASE + 1 * TILE, 1);
        issue_tile(kp, ld_offk, K_BASE + 2 * TILE, 2);
        issue_tile(kp, ld_offk, K_BASE + 3 * TILE, 3);
        issue_tile(vp, ld_offv, V_BASE + 1 * TILE, 1);
        {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int i = tid; i < TILE / 16; i += 64 * NW)
                *reinterpret_cast<u32x4*>(smem + V_BASE + 3 * TILE + i * 16) = z;
        }
        // the Q fragments (loaded before the first sweep, resident for both) and the prologue tiles have arrived
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+v"(qf[nq][kk]));
        wait_vmcnt<0>();
        barrier();

        // ---- S_0 = K_0 Q^T (not overlapped with anything)
        {
            const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb) {
                    const bf16x8 a = *(LDS_PTR(const bf16x8))(k_ptr[kk] + kb * 32 * (D * 2));
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        s_a[nq][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nq][kk], kk == 0 ? zero : s_a[nq][kb], 0, 0, 0);
                }
            if (BN > n_v) mask_tail(s_a, 0);
            if constexpr (!SAFE) {
                // fixed reference: the row max over the first key tile (key 0 is always valid)
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) {
                    float m0 = s_a[nq][0][0], m1 = s_a[nq][0][1];
#pragma unroll
                    for (int e = 2; e < 32; e += 2) {
                        m0 = fmaxf(m0, s_a[nq][e / 16][e % 16]);
                        m1 = fmaxf(m1, s_a[nq][(e + 1) / 16][(e + 1) % 16]);
                    }
                    mc_run[nq] = pair_max(fmaxf(m0, m1)) * c;
                    if constexpr (BASE2) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) nref[nq][r] = -mc_run[nq];
#pragma unroll
                        for (int e = 0; e < 32; ++e) s_a[nq][e / 16][e % 16] -= mc_run[nq];
                    }
                }
            }
        }
        barrier();           // K tile 0 is overwritten by the first DMA of the loop

        // One iteration; TB = t % 4 fixes every LDS buffer offset at compile time.
        //   s_c: scores of tile t (in, overwritten by its probabilities)   s_n: scores of tile t+1 (out)
        // Slot i (0..N_FR-1; N_FR = 32 for d = 128, 16 for d = 64) = the MFMAs fed by operand fragment
        // i (first the PV fragments, then as many QK fragments; NQ MFMAs each), the LDS reads of
        // fragment i+PF, and slice i of the softmax VALU work: slices 0-3 the row max, 4-5 the
        // reference / rescale factors, the others the 32 exponentials with their packing to bf16 and
        // the row sum.
        auto iteration = [&](auto tb_c, int t, f32x16 (&s_c)[NQ][NKB], f32x16 (&s_n)[NQ][NKB]) {
            constexpr int TB = decltype(tb_c)::value;
            constexpr int KN = (TB + 1) % NBUF;           // buffer of K tile t+1
            constexpr int VP = (TB + 3) % NBUF;           // buffer of V tile t-1
            // DMA of this iteration: K tile t+4 over K tile t, V tile t+2 over V tile t-2 (both last read
            // in iteration t-1).  Whole tiles take the short path: running scalar tile pointers, fixed
            // per-lane offsets, LDS destinations as immediates.
            if ((t + 5) * BN <= n_v) {
                static_for<0, CPW>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    lds_dma16_at<K_BASE + TB * TILE + j * (NW * 1024)>(k_dma, ld_k[j], dma_base);
                });
                static_for<0, CPW>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    lds_dma16_at<V_BASE + ((TB + 2) % NBUF) * TILE + j * (NW * 1024)>(v_dma, ld_v[j], dma_base);
                });
            } else {
                issue_tile(kp, ld_offk, K_BASE + TB * TILE, t + 4);
                issue_tile(vp, ld_offv, V_BASE + ((TB + 2) % NBUF) * TILE, t + 2);
            }
            k_dma += BN * D;
            v_dma += BN * D;
            constexpr int N_PV = NKB * 2 * NDB, N_QK = NKK * NKB, N_FR = N_PV + N_QK;
            constexpr int PF = 3, RING = 4;
            static_assert(N_FR == 32 || N_FR == 16, "slot plan below is written for 64-key tiles and d = 128 or 64");
            bf16x8 frag[RING];

            auto load_frag = [&](auto idx) {
                constexpr int i = decltype(idx)::value;
                if constexpr (i < N_PV) {
                    constexpr int kb = i / (2 * NDB), u = (i / NDB) % 2, db = i % NDB;
                    constexpr int off0 = VP * TILE + (kb * 32 + u * 16) * (D * 2);
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(v_ptr[db] + off0));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(v_ptr[db] + off0 + 8 * (D * 2)));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    frag[i % RING] = __builtin_bit_cast(bf16x8, av);
                } else if constexpr (i < N_FR) {
                    constexpr int j = i - N_PV, kk = j / 2, kb = j % 2;
                    frag[i % RING] = *(LDS_PTR(const bf16x8))(k_ptr[kk] + (KN * TILE + kb * 32 * (D * 2)));
                }
            };
            auto do_mfma = [&](auto idx, auto nq_c) {
                constexpr int i = decltype(idx)::value, nq = decltype(nq_c)::value;
                if constexpr (i < N_PV) {
                    constexpr int kb = i / (2 * NDB), u = (i / NDB) % 2, db = i % NDB;
                    const u32x4 pv = {p_io[nq][kb][u][0], p_io[nq][kb][u][1], p_io[nq][kb][u][2], p_io[nq][kb][u][3]};
                    o_acc[nq][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i % RING], __builtin_bit_cast(bf16x8, pv),
                                                                            o_acc[nq][db], 0, 0, 0);
                } else {
                    constexpr int j = i - N_PV, kk = j / 2, kb = j % 2;
                    if constexpr (kk == 0) {
                        const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                        s_n[nq][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i % RING], qf[nq][kk],
                                                                              (BASE2 && !SAFE) ? nref[nq] : zero, 0, 0, 0);
                    } else {
                        s_n[nq][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i % RING], qf[nq][kk], s_n[nq][kb], 0, 0, 0);
                    }
                }
            };

            // Softmax of tile t, slice by slice (anchored with empty asm statements: pure arithmetic
            // would otherwise drift out of the slot it is written in).
            float mx[NQ], mx2[NQ], mc_new[NQ], alpha[NQ], lsum[NQ], lsum2[NQ];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                mx[nq] = s_c[nq][0][0];
                mx2[nq] = s_c[nq][0][1];
                mc_new[nq] = SAFE ? 0.f : mc_run[nq]; alpha[nq] = 1.f; lsum[nq] = 0.f; lsum2[nq] = 0.f;
            }
            // Elements of the lane's 32 scores handled by exponential slot k (0..NX-1): [e_lo(k), e_lo(k+1)).
            // The work on an element is spread over consecutive slots so that no instruction needs a
            // result produced in its own slot: slot k-1 forms z = s*c - m, slot k takes exp2(z), slot k+1
            // adds it to the row sum and, once both halves of a pair exist, packs the pair to bf16.
            // SAFE: slots 0-3 row max, 4-5 reference and rescale factor, 6.. exponentials.  Otherwise the
            // exponentials start at slot 3 (not earlier: the packed pair q of this tile may replace that of
            // the previous tile only after the PV MFMAs of its group, which come d/32 slots per group in
            // the first half of the slots, have read it).
            constexpr int X0 = SAFE ? 6 : 3, NX = N_FR - X0;
            auto e_lo = [](int k) constexpr { return k <= 0 ? 0 : (k >= NX ? 32 : k * 32 / NX); };
            auto fma_of = [&](auto kc, auto nq_c) {
                constexpr int k = decltype(kc)::value, nq = decltype(nq_c)::value;
                if constexpr (BASE2 && !SAFE) return;             // the MFMA output already is s - reference
                static_for<e_lo(k), e_lo(k + 1)>([&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    float z = __builtin_fmaf(s_c[nq][e / 16][e % 16], c, -mc_new[nq]);
                    asm volatile("" : "+v"(z));
                    s_c[nq][e / 16][e % 16] = z;
                });
            };
            auto exp_of = [&](auto kc, auto nq_c) {
                constexpr int k = decltype(kc)::value, nq = decltype(nq_c)::value;
                static_for<e_lo(k), e_lo(k + 1)>([&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    float pe = __builtin_amdgcn_exp2f(s_c[nq][e / 16][e % 16]);
                    asm volatile("" : "+v"(pe));
                    s_c[nq][e / 16][e % 16] = pe;
                });
            };
            auto sum_pack_of = [&](auto kc, auto nq_c) {
                constexpr int k = decltype(kc)::value, nq = decltype(nq_c)::value;
                static_for<e_lo(k), e_lo(k + 1)>([&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    // row sum with plain adds, two chains (the dot-product instructions would take two
                    // values at a time, but they occupy the matrix pipe and stall the MFMA stream)
                    if constexpr (e % 2 == 0) {
                        lsum[nq] += s_c[nq][e / 16][e % 16];
                        asm volatile("" : "+v"(lsum[nq]));
                    } else {
                        lsum2[nq] += s_c[nq][e / 16][e % 16];
                        asm volatile("" : "+v"(lsum2[nq]));
                        constexpr int q = e / 2, kb = q / 8, u = (q % 8) / 4, j = q % 4;   // pair q = elements 2q, 2q+1
                        unsigned pk = pack_bf16(s_c[nq][kb][8 * u + 2 * j], s_c[nq][kb][8 * u + 2 * j + 1]);
                        asm volatile("" : "+v"(pk));
                        p_io[nq][kb][u][j] = pk;
                    }
                });
            };
            auto valu_slice = [&](auto idx, auto nq_c) {
                constexpr int i = decltype(idx)::value, nq = decltype(nq_c)::value;
                if constexpr (SAFE && i < 4) {                          // row max over the lane's 32 scores, two chains
#pragma unroll
                    for (int e = 8 * i; e < 8 * i + 8; e += 4) {
                        mx[nq] = fmaxf(fmaxf(mx[nq], s_c[nq][e / 16][e % 16]), s_c[nq][(e + 2) / 16][(e + 2) % 16]);
                        mx2[nq] = fmaxf(fmaxf(mx2[nq], s_c[nq][(e + 1) / 16][(e + 1) % 16]), s_c[nq][(e + 3) / 16][(e + 3) % 16]);
                    }
                } else if constexpr (SAFE && i == 4) {
                    // Move the reference only if the max grew by more than 2^8 (or there is none yet:
                    // -inf gives an infinite difference; a fully hidden tile gives -inf and no move).
                    const float mxc = pair_max(fmaxf(mx[nq], mx2[nq])) * c;
                    mc_new[nq] = (mxc - mc_run[nq] > 8.0f) ? mxc : mc_run[nq];
                } else if constexpr (SAFE && i == 5) {
                    alpha[nq] = __builtin_amdgcn_exp2f(mc_run[nq] - mc_new[nq]);      // 1 if unmoved, 0 on the first tile
                    fma_of(std::integral_constant<int, 0>{}, nq_c);
                } else if constexpr (!SAFE && i == X0 - 1) {
                    fma_of(std::integral_constant<int, 0>{}, nq_c);
                } else if constexpr (i >= X0) {                         // 32 exponentials over NX slots
                    constexpr int k = i - X0;
                    exp_of(std::integral_constant<int, k>{}, nq_c);
                    fma_of(std::integral_constant<int, k + 1>{}, nq_c);
                    sum_pack_of(std::integral_constant<int, k - 1>{}, nq_c);
                }
            };

            // ================= interleaved region: softmax(t) | PV(t-1), QK(t+1) =================
            static_for<0, PF>([&](auto i) { load_frag(i); });
            static_for<0, N_FR>([&](auto idx) {
                constexpr int i = decltype(idx)::value;
                static_for<0, NQ>([&](auto nq_c) { do_mfma(idx, nq_c); });
                load_frag(std::integral_constant<int, i + PF>{});
                static_for<0, NQ>([&](auto nq_c) { valu_slice(idx, nq_c); });
                __builtin_amdgcn_sched_barrier(0);
            });
            static_for<0, NQ>([&](auto nq_c) {
                constexpr int nq = decltype(nq_c)::value;
                sum_pack_of(std::integral_constant<int, NX - 1>{}, nq_c);
                if constexpr (SAFE) {
                    l_run[nq] = __builtin_fmaf(l_run[nq], alpha[nq], lsum[nq] + lsum2[nq]);
                    mc_run[nq] = mc_new[nq];
                } else {
                    l_run[nq] += lsum[nq] + lsum2[nq];
                }
            });
            // =====================================================================================

            // rescale O once PV(t-1) is in, if some lane moved its reference (rare after the first tiles)
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                if (SAFE && __builtin_amdgcn_ballot_w64(alpha[nq] != 1.0f) != 0) {
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o_acc[nq][db][r] *= alpha[nq];
                }
            }
            if ((t + 2) * BN > n_v) mask_tail(s_n, t + 1);     // S_{t+1} holds hidden keys

            if constexpr (NQ == 2) {
                // One wavefront per SIMD owns 512 registers, half of them accumulation registers that
                // only MFMAs (and loads) can address.  Pin what only MFMAs touch there - the O
                // accumulators and the Q fragments - so that the VALU-visible half is left for the scores.
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) {
#pragma unroll
                    for (int db = 0; db < NDB; ++db) asm volatile("" : "+a"(o_acc[nq][db]));
#pragma unroll
                    for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+a"(qf[nq][kk]));
                }
            }
            // Of the DMA batches in flight, all but the two newest (this iteration's, issued at its top,
            // and the previous one's) must have landed: K tile t+2 and V tile t, which iteration t+1 reads.
            wait_vmcnt<4 * CPW>();
            barrier();
        };

        // The loop runs over tiles 0 .. nt (the extra one only completes PV(nt-1): its scores are all
        // hidden, so its probabilities are zero), unrolled by four so that buffer offsets are
        // immediates and the score / probability registers alternate roles without copies.
        // (the loop is left right after iteration nt, wherever in the group of four that falls)
        for (int t = 0; t <= nt; t += 4) {
            iteration(std::integral_constant<int, 0>{}, t, s_a, s_b);
            if (t == nt) break;
            iteration(std::integral_constant<int, 1>{}, t + 1, s_b, s_a);
            if (t + 1 == nt) break;
            iteration(std::integral_constant<int, 2>{}, t + 2, s_a, s_b);
            if (t + 2 == nt) break;
            iteration(std::integral_constant<int, 3>{}, t + 3, s_b, s_a);
        }
        wait_vmcnt<0>();        // no DMA may outlive the workgroup's LDS
    };
    sweep(std::false_type{});
    {
        // A row whose sum left the safe range (a later score exceeded the first tile's max by more
        // than ~2^64, or non-finite input) or whose accumulators are not finite makes the whole
        // workgroup redo the item with the running max (weights <= 2^8 there).
        bool bad = p.redo_always != 0;               // test switch: every item takes the second sweep
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            bad |= !(pair_sum(l_run[nq]) < 1.8446744e19f);
            // Weights of up to 2^64 times large finite V entries can overflow the accumulators while the
            // row sum stays in range: inf * 0 and NaN * 0 are NaN, any finite value * 0 is 0.
            float t = 0.f;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) t = __builtin_fmaf(o_acc[nq][db][r], 0.0f, t);
            bad |= !(t == 0.f);
        }
        const bool wave_bad = __builtin_amdgcn_ballot_w64(bad) != 0;
        barrier();                                   // every wavefront is done with the LDS tiles and its DMA
        LDS_PTR(volatile int) flags = (LDS_PTR(volatile int))smem;
        if (lane == 0) flags[wave] = wave_bad ? 1 : 0;
        barrier();
        int any = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) any |= flags[w];
        barrier();                                   // flags are read before the redo's DMA reuses their bytes
        if (__builtin_amdgcn_readfirstlane(any)) sweep(std::true_type{});
    }

    // ---- epilogue: normalise, write out and lse.  The lane's row is formed from a copy of its index
    // that the compiler cannot trace back, or it would form the store addresses before the sweep and
    // carry them through it in registers the loop has no room for.
    int li_e = li;
    asm volatile("" : "+v"(li_e));
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float l_tot = pair_sum(l_run[nq]);
        const float inv = 1.0f / l_tot;
        const int64_t row = q_row0 + nq * 32 + li_e;
        if (row < Sq) {
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 o4 = {o_acc[nq][db][4 * a] * inv, o_acc[nq][db][4 * a + 1] * inv,
                                o_acc[nq][db][4 * a + 2] * inv, o_acc[nq][db][4 * a + 3] * inv};
                    if (store_bf16) {
                        const u32x2 h2 = {pack_bf16(o4[0], o4[1]), pack_bf16(o4[2], o4[3])};
                        *reinterpret_cast<u32x2*>(oph + row * D + db * 32 + a * 8 + 4 * lh) = h2;
                    } else {
                        *reinterpret_cast<f32x4*>(op + (row - row_sub) * D + db * 32 + a * 8 + 4 * lh) = o4;
                    }
                }
            if (lh == 0) lp[row - row_sub] = mc_run[nq] * 0.6931471805599453f + __logf(l_tot);
        }
    }
    }   // next work item

    // The last workgroup to leave puts both counters back to zero for the next launch that uses this
    // workspace (launches sharing a workspace are ordered on one stream).  Every workgroup has made
    // its last fetch before it counts itself out, so nobody fetches after the reset.
    if (!direct && tid == 0) {
        __threadfence();
        if (atomicAdd(p.counter + 1, 1) == (int)gridDim.x - 1) {
            __hip_atomic_store(p.counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.counter + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Folds the key-range partials of the cut tiles into out/lse (in place): per row,
// L = ln sum_p exp(lse_p), out = sum_p exp(lse_p - L) out_p.  One group of d/4 lanes (half or a
// quarter of a wavefront) per row, so a row's lse is read by all its lanes before one of them
// overwrites it.
template <int D>
__global__ __launch_bounds__(256) void tail_merge_kernel(const AttnParams p, int n_tail) {
    constexpr int M = 256, LPR = D / 4, RPB = 256 / LPR;      // lanes per row, rows per workgroup
    const int tile = p.n_full + blockIdx.x / (M / RPB);
    const int r_in = (blockIdx.x % (M / RPB)) * RPB + (threadIdx.x / LPR);
    const int c4 = threadIdx.x % LPR;
    const int bh = tile / p.tiles_per_head;
    const int q_tile = tile - bh * p.tiles_per_head;
    const int b = bh / p.Hg, h = bh - b * p.Hg;
    const int64_t row = (int64_t)q_tile * M + r_in;
    if (row >= p.Sq) return;
    float* lp = p.lse + (int64_t)b * p.l_bs + (int64_t)h * p.l_hs + row;
    // fp32 out: part 0 sits in out/lse and parts 1.. in the workspace; bf16 out: all parts in the workspace
    const int n_ws = p.out_bf16 ? p.split : p.split - 1;
    const int64_t slot0 = (int64_t)(tile - p.n_full) * n_ws;
    // one pass with a running reference (the parts of a cut tile are never empty: lse is finite)
    float m = -INFINITY, tot = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < p.split; ++j) {
        float lj;
        float4 xj;
        if (j == 0 && !p.out_bf16) {
            lj = *lp;
            xj = reinterpret_cast<const float4*>(p.out + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs + row * D)[c4];
        } else {
            const int64_t slot = slot0 + (p.out_bf16 ? j : j - 1);
            lj = p.part_lse[slot * M + r_in];
            xj = reinterpret_cast<const float4*>(p.part_out + (slot * M + r_in) * D)[c4];
        }
        const float m_new = fmaxf(m, lj);
        const float a_old = __expf(m - m_new);          // 0 on the first part
        const float w = __expf(lj - m_new);
        acc.x = acc.x * a_old + w * xj.x; acc.y = acc.y * a_old + w * xj.y;
        acc.z = acc.z * a_old + w * xj.z; acc.w = acc.w * a_old + w * xj.w;
        tot = tot * a_old + w;
        m = m_new;
    }
    const float inv = 1.0f / tot;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    if (p.out_bf16) {
        __bf16* oh = reinterpret_cast<__bf16*>(p.out) + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs + row * D;
        reinterpret_cast<uint2*>(oh)[c4] = make_uint2(pack_bf16(acc.x, acc.y), pack_bf16(acc.z, acc.w));
    } else {
        reinterpret_cast<float4*>(p.out + (int64_t)b * p.o_bs + (int64_t)h * p.o_hs + row * D)[c4] = acc;
    }
    if (c4 == 0) *lp = m + __logf(tot);
}

template <int D, int NQ, bool BASE2>
static hipError_t launch_sp(AttnParams p, int BH, float* ws, int64_t ws_slots, hipStream_t st) {
    constexpr int smem = 2 * 4 * 64 * D * 2;        // 128 KB (d = 128) or 64 KB
    constexpr int M = 256;
    auto kern = attn_fwd_sp_kernel<D, NQ, BASE2>;
    static KernelSetup setup;
    int n_cu = 0;
    {
        hipError_t e = setup.ensure(reinterpret_cast<const void*>(kern), smem, &n_cu);
        if (e != hipSuccess) return e;
    }
    const TailPlan t = plan_tail(p.Sq, BH, p.n_v, n_cu);
    const int64_t slots = tail_slots(t, p.out_bf16 != 0);
    if (ws == nullptr || slots > ws_slots) return hipErrorInvalidValue;
    // no key range may be empty or start off a 64-key boundary
    if (t.split > 1) {
        if (t.split > kMaxSplit || t.part_off[0] != 0 || t.part_off[t.split] != p.n_v) return hipErrorInvalidValue;
        for (int j = 0; j < t.split; ++j)
            if (t.part_off[j + 1] <= t.part_off[j] || t.part_off[j] % 64 != 0) return hipErrorInvalidValue;
    }
    p.tiles_per_head = t.tiles_per_head;
    p.split = t.split;
    p.n_cut = (int)t.n_cut;
    p.n_full = (int)(t.n_tiles - t.n_cut);
    for (int j = 0; j <= kMaxSplit; ++j) p.part_off[j] = t.part_off[j];
    p.part_out = slots ? ws : nullptr;
    p.part_lse = slots ? ws + slots * (M * D) : nullptr;
    p.counter = reinterpret_cast<int*>(ws + ws_slots * kSlotFloats);     // two ints behind the slots, zero between launches
    const int64_t items = p.n_full + t.n_cut * t.split;
    p.n_items = (int)items;
    const unsigned grid = (unsigned)(items < n_cu ? items : n_cu);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512 / NQ), smem, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || t.split <= 1) return e;
    hipLaunchKernelGGL(tail_merge_kernel<D>, dim3((unsigned)(t.n_cut * (M / (1024 / D)))), dim3(256), 0, st, p, (int)t.n_cut);
    return hipGetLastError();
}

hipError_t launch_attn_fwd_sp(const AttnParams& p, int BH, int D, float* ws, int64_t ws_slots, hipStream_t st) {
    if (D == 64)
        return p.base2 ? launch_sp<64, 1, true>(p, BH, ws, ws_slots, st) : launch_sp<64, 1, false>(p, BH, ws, ws_slots, st);
    return p.base2 ? launch_sp<128, 1, true>(p, BH, ws, ws_slots, st) : launch_sp<128, 1, false>(p, BH, ws, ws_slots, st);
}

}  // namespace pda
