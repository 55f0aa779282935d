// Internal declarations shared by the translation units of libpipedit_attn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace pda {

// One-time, per-device launch setup of a kernel that needs more than the default dynamic LDS size:
// sets the attribute on the current device the first time the kernel is launched there and
// returns that device's CU count through n_cu.  One instance per kernel (function-local static).
struct KernelSetup {
    static constexpr int MAX_DEV = 64;
    std::atomic<int> cu[MAX_DEV] = {};
    hipError_t ensure(const void* kern, int smem_bytes, int* n_cu) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool cached = dev >= 0 && dev < MAX_DEV;
        int v = cached ? cu[dev].load(std::memory_order_acquire) : 0;
        if (v == 0) {   // two threads may both get here: setting the attribute twice is harmless
            if ((e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes)) != hipSuccess) return e;
            if ((e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
            if (cached) cu[dev].store(v, std::memory_order_release);
        }
        if (n_cu) *n_cu = v;
        return hipSuccess;
    }
};

// One attention launch over Hg heads of B batches.  Strides are in elements; a head group of a
// compact [B,H,S,d] tensor is addressed by offsetting the base pointers and keeping the full
// tensor's batch stride.
struct AttnParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    float* out;
    float* lse;
    int64_t Sq;
    int64_t n_v;            // number of valid keys (kv_valid_len)
    int64_t q_bs, q_hs;     // q batch / head stride
    int64_t kv_bs, kv_hs;   // k and v batch / head stride
    int64_t o_bs, o_hs;     // out batch / head stride
    int64_t l_bs, l_hs;     // lse batch / head stride
    int Hg;                 // heads in this launch
    float scale;            // softmax scale
    float scale_log2e;      // scale * log2(e)
    // Work items of the software-pipelined kernel, taken in index order by persistent workgroups.
    // Items [0, n_full) are whole 256-row query tiles (tile = item; head = tile / tiles_per_head).
    // Every later tile is cut into `split` key ranges [part_off[j], part_off[j+1]), one item each
    // (item = n_full + part * n_cut + cut tile), so that the end of the launch is made of short items;
    // part 0 writes out/lse, parts >= 1 write normalised partials to part_out/part_lse, which a
    // merge pass folds into out/lse.  split <= 1: no cut.
    int tiles_per_head;
    int n_full;
    int split;
    int64_t part_off[17];   // first key of each range (multiples of 64); part_off[split] = n_v
    float* part_out;        // [(tile - n_full) * (split - 1) + part - 1][256][d]
    float* part_lse;        // [(tile - n_full) * (split - 1) + part - 1][256]
    int n_cut;              // number of cut tiles (the last n_cut of the launch)
    int n_items;            // n_full + n_cut * split
    int* counter;           // two ints, zero between launches: next work item, workgroups that have finished
    int out_bf16;           // software-pipelined kernel: `out` points to bf16 elements (same element strides)
    int base2;              // scores are already in log2 units: weights 2^(q.k), scale_log2e == 1
    int redo_always;        // software-pipelined kernel: sweep every item a second time with the running max (testing aid)
};

// Tail plan of the software-pipelined kernel (256-row query tiles, one persistent
// workgroup per CU taking items in order).  Whole tiles are long items (a 119 056-key sweep takes
// 3 ms), the XCDs run at different speeds, and a launch ends when the last item does; so the
// `rem` = n_tiles mod n_cu tiles that do not fill a round of whole tiles are cut into `split` key
// ranges, short items that the workgroups pick up as they run out of whole tiles.  Measured on
// the device: about three part items per CU balance the end of a long launch; every part pays a
// prologue, a partial store and its share of the merge, so parts are kept at 100 key tiles or more
// (50 where that gives no more than 4 ranges).  Rule:
//     split = round(3 * n_cu / rem), at least 2, at most the smallest of
//             16, max(nt / 100, min(nt / 50, 4)) (nt = key tiles of a whole sweep), n_v / 512,
//             1 + (9 * n_cu / 4) / rem   (workspace: the parts beyond the first must fit),
//     lowered until the last range is not empty; uncut if that leaves less than 2 or rem = 0.
// Where the parts are short and the CUs become free together, parts run in rounds like tiles do,
// and ONE round of parts is best: split = floor(n_cu / rem) under the same caps except the one on
// the part length.  That is the plan of a launch with fewer tiles than CUs (one head of a short
// clip, the unit PipeSP pipelines, would otherwise leave CUs without work for its whole duration;
// measured: 38 tiles of 150 key tiles, split 6: 0.081 ms instead of 0.181 ms) and of sweeps of
// under 200 key tiles whose left-over tiles fill at most half the machine (measured: 10 heads x
// 9 600 tokens, rem = 124: 0.502 / 0.428 / 0.451 / 0.442 ms for split 1 / 2 / 3 / 4).
// Where the left-over tiles fill more than half the machine and at most three rounds of whole
// tiles precede them, no equal cut within the workspace balances the end (210 left-over tiles in
// 3 ranges are 630 parts: 2.5 rounds, which end when 3 would).  Such tiles are cut UNEQUALLY: a
// long first range of a fraction A of the keys, taken by rem CUs, and split-1 short ranges, which
// the other n_cu - rem CUs work off meanwhile, k each: k = ceil(rem (split-1) / (n_cu - rem)),
// A = k / (k + split - 1) (both kinds of CU then finish together), split = 4 after one round of
// whole tiles, else 3, within the workspace cap and with short ranges of at least 1024 keys
// (measured, one head at S = 119 056 = 256 + 210 tiles: 5.78 -> 5.47 ms; 5 x 36 000: 2.64 -> 2.55).
// After four or more rounds of whole tiles the CUs do not become free together, items are handed
// out as CUs ask for them, and what is left idle at the end is about half of the items started
// last.  There the ranges (2 to 6 of them) get DECREASING sizes, each 5/8 of the one before, range
// 0 first: the items started last are the shortest (measured, 3-head group at S = 119 056, five
// ranges of 41 / 26 / 16 / 10 / 6 % instead of 20 % each: 16.53 -> 16.43 ms; 6 heads, three
// ranges of 50 / 31 / 19 %: 32.98 -> 32.85 ms); kept equal if the last range would fall under
// 50 key tiles.
// A pure function of (Sq, number of (batch, head) pairs, valid keys, CU count): the cut tiles are
// the last n_cut of the launch's n_tiles tiles in (batch, head, query tile) order.
constexpr int kMaxSplit = 16;
struct TailPlan {
    int tiles_per_head;
    int64_t n_tiles;
    int64_t n_cut;          // 0 if no tile is cut
    int split;              // 1 if no tile is cut
    int64_t part_off[kMaxSplit + 1];   // range j of a cut tile = keys [part_off[j], part_off[j+1]); multiples of 64 up to
                                       // part_off[split] = n_v; entries beyond split are n_v as well
};
inline int64_t max_extra_slots(int n_cu) { return (int64_t)n_cu * 9 / 4; }
inline int64_t part_keys_for(int64_t n_v, int s) { return ((n_v + s - 1) / s + 63) / 64 * 64; }
inline TailPlan plan_tail(int64_t Sq, int BH, int64_t n_v, int n_cu) {
    TailPlan t{};
    t.tiles_per_head = (int)((Sq + 255) / 256);
    t.n_tiles = (int64_t)t.tiles_per_head * BH;
    t.split = 1;
    const int64_t rem = t.n_tiles % n_cu;
    bool one_round = false;
    if (rem) {
        const int64_t nt = (n_v + 63) / 64;
        // One round of parts (n_cu / rem ranges per tile) where the parts are short and start together:
        // a launch of fewer tiles than CUs, or sweeps of under 200 key tiles whose left-over tiles
        // fill at most half the machine.  Otherwise about three rounds of parts, round(3 n_cu / rem),
        // of at least 100 key tiles each (at least 50 where that gives no more than 4 ranges).
        one_round = t.n_tiles < n_cu || (nt < 200 && 2 * rem <= n_cu);
        int64_t s_max = kMaxSplit;
        if (!one_round) {
            int64_t by_len = nt / 50 < 4 ? nt / 50 : 4;
            if (nt / 100 > by_len) by_len = nt / 100;
            if (by_len < s_max) s_max = by_len;
        }
        if (n_v / 512 < s_max) s_max = n_v / 512;
        if (1 + max_extra_slots(n_cu) / rem < s_max) s_max = 1 + max_extra_slots(n_cu) / rem;
        int64_t s = one_round ? n_cu / rem : (6 * (int64_t)n_cu + rem) / (2 * rem);
        if (s < 2 && !one_round) s = 2;
        if (s > s_max) s = s_max;
        while (s >= 2 && (s - 1) * part_keys_for(n_v, (int)s) >= n_v) --s;   // the last range must not be empty
        if (s >= 2) t.split = (int)s;
    }
    for (int j = 0; j <= kMaxSplit; ++j) t.part_off[j] = n_v;
    if (t.split > 1) {
        t.n_cut = rem;
        const int64_t pk = part_keys_for(n_v, t.split);
        for (int j = 0; j < t.split; ++j) t.part_off[j] = j * pk;
        // decreasing ranges after four or more rounds of whole tiles: weights 8^(s-1-j) 5^j
        if (!one_round && t.n_tiles >= 4 * (int64_t)n_cu && t.split <= 6) {
            int64_t w[6], total = 0, cum = 0, off[7];
            for (int j = 0; j < t.split; ++j) {
                w[j] = 1;
                for (int i = 0; i < t.split - 1 - j; ++i) w[j] *= 8;
                for (int i = 0; i < j; ++i) w[j] *= 5;
                total += w[j];
            }
            off[0] = 0;
            for (int j = 1; j < t.split; ++j) { cum += w[j - 1]; off[j] = n_v * cum / total / 64 * 64; }
            off[t.split] = n_v;
            bool ok = n_v - off[t.split - 1] >= 3200;
            for (int j = 0; j < t.split; ++j) ok = ok && off[j + 1] > off[j];
            if (ok) for (int j = 0; j < t.split; ++j) t.part_off[j] = off[j];
        }
    }
    // unequal cut: many left-over tiles after at most three rounds of whole tiles
    if (rem && 2 * rem > n_cu && t.n_tiles < 4 * (int64_t)n_cu && t.n_tiles > n_cu) {
        int64_t s = t.n_tiles < 2 * (int64_t)n_cu ? 4 : 3;
        if (1 + max_extra_slots(n_cu) / rem < s) s = 1 + max_extra_slots(n_cu) / rem;
        for (; s >= 2; --s) {
            const int64_t k = (rem * (s - 1) + (n_cu - rem) - 1) / (n_cu - rem);
            const int64_t first = ((n_v * k / (k + s - 1) + n_v / 100) / 64 + 1) * 64;
            if (first >= n_v) continue;
            const int64_t part = ((n_v - first + (s - 2)) / (s - 1) + 63) / 64 * 64;
            if (part < 1024 || first + (s - 2) * part >= n_v) continue;    // short ranges too short, or the last one empty
            t.split = (int)s;
            t.n_cut = rem;
            for (int j = 0; j <= kMaxSplit; ++j) t.part_off[j] = j == 0 ? 0 : (j < s ? first + (j - 1) * part : n_v);
            break;
        }
    }
    return t;
}
// One workspace slot holds one key-range partial of a cut tile: 256 x 128 values + 256 lse.
// A workspace of n slots is n * kSlotFloats floats followed by kCounterFloats floats that hold the
// kernel's two work counters (zero whenever no launch is running on it).
constexpr size_t kSlotFloats = 256 * 128 + 256;
constexpr size_t kCounterFloats = 64;
// Slots a launch needs: parts 1.. of every cut tile (part 0 goes to out/lse), or all parts when
// out is bf16 (the merge pass then needs part 0 in fp32 as well).
inline int64_t tail_slots(const TailPlan& t, bool out_bf16) {
    return t.split > 1 ? t.n_cut * (out_bf16 ? t.split : t.split - 1) : 0;
}
// Largest slot count any launch can need on a device with n_cu compute units.
inline int64_t max_tail_slots(int n_cu, bool out_bf16) {
    return max_extra_slots(n_cu) + (out_bf16 ? n_cu - 1 : 0);
}

// Enqueue the forward kernel for B*Hg = BH (batch, head) pairs.  variant selects a tiling (0 = the
// software-pipelined kernel for d = 128; 1, 2 = reference tilings; 3 = 0 with its running-max sweep
// forced on every item).  ws / ws_slots: device workspace for the key-range partials of the
// software-pipelined kernel and its capacity in slots of kSlotFloats floats; a launch that needs
// more returns hipErrorInvalidValue (the caller sizes it with plan_tail / tail_slots).
hipError_t launch_attn_fwd(const AttnParams& p, int BH, int D, int variant, float* ws, int64_t ws_slots, hipStream_t st);

// Software-pipelined kernel for d = 128 (attn_fwd_sp.hip); p.n_v >= 1, p.scale_log2e > 0.
hipError_t launch_attn_fwd_sp(const AttnParams& p, int BH, int D, float* ws, int64_t ws_slots, hipStream_t st);

// Does this (d, variant, valid key count) take the software-pipelined kernel (and so possibly a workspace)?
inline bool uses_sp_kernel(int D, int variant, int64_t n_v) { return (D == 128 || D == 64) && n_v > 0 && (variant == 0 || variant == 3); }

// CU count of the current device (cached per device).
hipError_t device_cu_count(int* n_cu);

struct MergeParams {
    const float* part[16];
    const float* lse[16];
    float* out;
    float* lse_out;         // nullable
    int64_t rows;
    int n;
};
hipError_t launch_merge(const MergeParams& p, int d, hipStream_t st);

// Copy n floats (n % 4 == 0, 16-byte aligned) on a stream: the hand-off op of the head-chunk pipeline.
hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st);

// Algorithm 1 steps 10-13 in one pass: hidden[r, i*h + j, :] = chunk[j][r, i, :].
struct PostParams {
    const float* chunk[64];  // h device pointers
    float* hidden;           // [rows, n*h, D]
    int64_t rows;
    int64_t row_stride4;     // distance between rows of a chunk, in float4s
    int h, n, D4;            // D4 = D / 4
};
hipError_t launch_postprocess(const PostParams& p, hipStream_t st);

// Hand-off of hg heads [hg, S, d] (global heads h0.. of H = n*h) into a token-major [S, H, d]
// buffer; arrival != 0 places head i*h+j at slot j*n+i (PipeSP's arrival order), else at i*h+j.
hipError_t launch_scatter_heads(const float* src, float* dst, int64_t S, int d, int hg, int H, int h0,
                                int h, int n, int arrival, hipStream_t st);

// Token-major fp32 [B,S,H,d] -> head-major bf16 [B,H,S,d] (d = 64 or 128), optional unit-RMS vectors,
// every element times premul before the rounding.
hipError_t launch_pack(const float* x, void* y, int B, int64_t S, int H, int d, int unit_rms, float premul, hipStream_t st);

// MFMA rate probes (probe.hip): n_cu workgroups x 8 wavefronts, each wavefront issues about 8*iters
// MFMAs (32x32x16 bf16) on fragments read from src (n_frag 16-byte fragments); mix 0 = MFMAs only,
// 1..3 = with the other instruction classes of the attention loop added; sink: >= 512 floats.
hipError_t launch_mfma_rate(const void* src, int64_t n_frag, int64_t iters, int n_cu, int mix, float* sink, hipStream_t st);

}  // namespace pda
