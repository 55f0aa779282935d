// Internal declarations shared by the translation units of libpipedit_attn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pda {

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
};

// Enqueue the forward kernel for B*Hg = BH (batch, head) pairs.  variant selects a tiling (0 = default).
hipError_t launch_attn_fwd(const AttnParams& p, int BH, int D, int variant, hipStream_t st);

// Ping-pong scheduled kernel for d = 128 (attn_fwd_pp.hip); p.n_v >= 1.
hipError_t launch_attn_fwd_pp(const AttnParams& p, int BH, int mode, hipStream_t st);

// Software-pipelined kernel for d = 128 (attn_fwd_il.hip); p.n_v >= 1, p.scale_log2e > 0.
hipError_t launch_attn_fwd_il(const AttnParams& p, int BH, hipStream_t st);

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

}  // namespace pda
