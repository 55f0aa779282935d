/*
 * libpipedit_attn: the attention hot path of PipeDiT video-DiT inference on MI355X (gfx950).
 *
 * C ABI.  Every pointer is a DEVICE pointer unless the comment says "host".
 * The caller owns every tensor.  The library itself keeps one device workspace
 * per (device, stream) for the attention kernel: its work counters and
 * the key-range partials of cut query tiles (see pda_attn_tail_plan).  It is
 * allocated once, the first time that kernel is launched on the stream, with
 * the largest size any launch can need
 * on that device (831 slots of 132 096 bytes = 110 MB with 256 compute units);
 * it never grows and is kept until the process ends, so after that first call
 * per stream the attention entry points neither allocate nor free nor
 * synchronise.  Work enqueued on one stream shares that stream's workspace,
 * which is safe because a stream runs its work in order; calls on different
 * streams use different workspaces.  If that one allocation fails the call
 * returns PDA_ERR_NOMEM and launches nothing.  All tensors are
 * compact row-major for exactly the sizes passed:
 *
 *     q    [B, H, Sq,  d]  bf16        k, v [B, H, Skv, d]  bf16
 *     out  [B, H, Sq,  d]  fp32        lse  [B, H, Sq]      fp32 (natural log)
 *
 * which is the head-major layout of Algorithm 1's input (Q in R^{B x h x S x D};
 * Q[:, j, :, :] is one head).  d must be 64 or 128.  Base pointers must be
 * 16-byte aligned.
 *
 * Errors: every entry point returns a pda_status; nothing throws or aborts.
 * Arguments are validated before any device work, so the error paths can be
 * exercised on a machine without a GPU.  pda_last_error() gives the message of
 * the calling thread's last failure.
 *
 * Asynchrony: kernels are enqueued on the given hipStream_t (passed as void*;
 * NULL is the default stream) and the call returns without waiting, except
 * where stated.  Results are deterministic run to run (no atomics in any
 * reduction).
 */
#ifndef PIPEDIT_ATTN_H
#define PIPEDIT_ATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PDA_OK = 0,
    PDA_ERR_INVALID_ARG = 1, /* null pointer, negative size, kv_valid_len > Skv, n < 1, ... */
    PDA_ERR_UNSUPPORTED = 2, /* d not in {64,128}, n > PDA_MAX_PARTIALS, misaligned pointer, size overflow */
    PDA_ERR_HIP = 3,         /* a HIP runtime call failed; see pda_last_error() */
    PDA_ERR_NOMEM = 4        /* the one-time device workspace of a stream could not be allocated */
} pda_status;

#define PDA_MAX_PARTIALS 16

/*
 * Attention forward for one head group or one query range: the black-box call
 * of Algorithm 1, step 3 (attention(Q[:,j], K[:,j], V[:,j], mask[:,j])) and of
 * the Attention Co-processing section (Attn(Q,K,V)), taken as scaled
 * dot-product softmax attention.  For every (b, h) and query row i:
 *
 *     s_j = scale * <q_i, k_j>  for j < kv_valid_len;   keys j >= kv_valid_len are hidden
 *     lse_i = ln sum_j exp(s_j),      out_i = sum_j exp(s_j - lse_i) * v_j
 *
 * The mask of Algorithm 1 is reduced to that key-padding tail.  0 <=
 * kv_valid_len <= Skv; kv_valid_len == Skv means no mask; kv_valid_len == 0
 * writes out = 0 and lse = -inf (an empty share of the keys).  K/V rows at or
 * beyond kv_valid_len are never read.
 *
 * q_offset (>= 0) is the global index of this call's first query row inside
 * the full sequence when the call covers a query range; attention here is
 * full (non-causal), so it does not change any value and is only validated.
 * The caller places the range's rows by offsetting out/lse itself.
 *
 * Arithmetic: bf16 x bf16 products accumulated in fp32 on the matrix cores,
 * softmax statistics in fp32, probabilities rounded to bf16 before the PV
 * product.  Finite inputs give finite results as long as
 * kv_valid_len * 2^8 * max|v| stays below the fp32 range (|v| up to 2^100 at
 * any supported length); scores of any finite magnitude are handled.
 * Sq == 0 or B*H == 0 is a successful no-op.
 */
int pda_attn_fwd(const void* q, const void* k, const void* v, float* out, float* lse,
                 int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                 int64_t kv_valid_len, int64_t q_offset, void* stream);

/*
 * pda_attn_fwd on views: the same computation with explicit batch and head strides (in
 * ELEMENTS) for q, k/v (shared), out and lse, so that a query range or a key chunk of larger
 * tensors is passed without a copy (Attention Co-processing shares; Ring-Attention style key
 * chunks): q = Q + q_offset*d with Q's strides, k = K + chunk_start*d with K's strides, and so on.
 * Rows stay compact (consecutive rows are d elements apart).  Strides of q and k/v must be
 * multiples of 8, of out multiples of 4 (16-byte alignment of every row); the head stride of out
 * must be >= Sq*d and of lse >= Sq, and with B > 1 a batch must not overlap the next one
 * (batch stride >= (H-1)*head stride + extent of one head), for out and lse, which are written.
 * pda_attn_fwd is this call with the strides of compact [B,H,S,d] tensors.
 */
int pda_attn_fwd_strided(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d,
                         int64_t q_batch_stride, int64_t q_head_stride,
                         int64_t kv_batch_stride, int64_t kv_head_stride,
                         int64_t out_batch_stride, int64_t out_head_stride,
                         int64_t lse_batch_stride, int64_t lse_head_stride,
                         float scale, int64_t kv_valid_len, int64_t q_offset, void* stream);

/*
 * pda_attn_fwd for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments, same arithmetic and the
 * same work plan as pda_attn_fwd, but the key-range partials of cut query tiles (see
 * pda_attn_tail_plan) go to a fixed buffer inside the library instead of the stream's workspace,
 * and the call allocates, frees and synchronises nothing.  (Its first call on a device looks up
 * the buffer's address, once; a caller that captures graphs makes one call before capturing.)
 * The buffer is a device array of PDA_NOALLOC_SCRATCH_BYTES bytes (PDA_NOALLOC_MAX_SLOTS partial
 * slots of 132 096 bytes) that every GPU the library runs on holds from the time the library is
 * loaded until the process ends.  A launch whose plan needs more slots than that returns
 * PDA_ERR_UNSUPPORTED and launches nothing (with 256 compute units no fp32-output launch needs
 * more than 576 slots, so nothing is rejected there).  All calls on one GPU share the one buffer,
 * whatever their stream: calls whose execution may overlap on a GPU race on it and must be
 * ordered by the caller (one stream, or events).  The buffer also holds the kernel's two work
 * counters, which are zero when the library is loaded and which every launch leaves at zero;
 * every partial slot a launch reads was written by the same launch first.
 */
#define PDA_NOALLOC_MAX_SLOTS 576
#define PDA_NOALLOC_SCRATCH_BYTES 76087552 /* 576 * (256*128 + 256) * 4 for the partials + 256 for the work counters */
int pda_attn_fwd_noalloc(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, int64_t q_offset, void* stream);

/*
 * How an attention launch over B*H (batch, head) pairs is cut into work items (host only;
 * every pointer below is a HOST pointer; no device work).  The kernel takes 256-row query tiles,
 * one workgroup per compute unit at a time, so tiles run in rounds of n_cu.  The last n_cut tiles
 * (in (batch, head, query tile) order: the partly filled last round; all tiles of a launch
 * with fewer tiles than compute units; none where the key ranges would get too short to pay)
 * are each computed as `split` (2..PDA_MAX_KEY_RANGES) partial attentions over consecutive key
 * ranges, range j = keys [part_offsets[j], part_offsets[j+1]) with boundaries at multiples of 64,
 * and merged with the formula of pda_attn_merge; all other tiles are swept in one pass.  The
 * ranges are equal, or a long first one and short others (many left-over tiles after one to three
 * rounds of whole tiles), or of decreasing size (after four or more rounds), whichever balances
 * the end of the launch better.  Hence two launches agree bit for bit on every row that lies in
 * an uncut tile of both, and to the rounding of the probabilities on the others.
 * n_cu: compute units of the device (0 = ask the current device).  Outputs (any may be NULL):
 * n_tiles; n_cut (0 = nothing is cut); split (1 = nothing is cut); part_offsets, a HOST array of
 * PDA_MAX_KEY_RANGES + 1 values (part_offsets[0] = 0, entries from index split on are
 * kv_valid_len); workspace_slots, the number of 132 096-byte partial slots the launch uses (fp32
 * out; never more than 9/4 per compute unit; a d = 64 launch fills half of each slot).  Empty key
 * sets are never cut.
 */
#define PDA_MAX_KEY_RANGES 16
int pda_attn_tail_plan(int B, int H, int64_t Sq, int64_t kv_valid_len, int d, int n_cu,
                       int64_t* n_tiles, int64_t* n_cut, int* split, int64_t* part_offsets, int64_t* workspace_slots);

/*
 * Testing aid: pda_attn_fwd (no q_offset) with an explicit choice of kernel.
 * variant 0 = what pda_attn_fwd runs; 1, 2 = two plain reference tilings of the same MFMA
 * formulation (128 and 256 query rows per workgroup, register-staged double buffering, running
 * max); 3 = variant 0 with its second, running-max sweep forced on every work item.  All compute
 * the same function to rounding.
 */
int pda_attn_fwd_variant(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, int variant, void* stream);

/*
 * pda_attn_fwd with a bf16 output, for results that go straight on to the next projection and not
 * through pda_attn_merge (which takes fp32 partials): out is [B,H,Sq,d] bf16, rounded to nearest
 * even from the fp32 result; lse stays fp32.  Everything else as pda_attn_fwd.
 */
int pda_attn_fwd_bf16out(const void* q, const void* k, const void* v, void* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, void* stream);

/*
 * pda_attn_fwd for callers that fold the softmax scale into Q where Q is produced (for instance
 * pda_pack_heads with premul = scale * log2(e), which costs no extra rounding there): the scores
 * s_j = <q_i, k_j> are taken to be in units of log2, i.e.
 *
 *     lse_i = ln sum_j 2^(s_j),      out_i = sum_j 2^(s_j) v_j / sum_j 2^(s_j)
 *
 * which is pda_attn_fwd with scale = ln 2 evaluated exactly.  The kernel then needs no arithmetic
 * between the matrix product and the exponential.  Arguments as pda_attn_fwd.
 */
int pda_attn_fwd_base2(const void* q, const void* k, const void* v, float* out, float* lse,
                       int B, int H, int64_t Sq, int64_t Skv, int d, int64_t kv_valid_len, void* stream);

/*
 * Exact merge of n partial attentions computed over disjoint key sets (the
 * recombination a Ring-Attention style key split needs, and what re-joins
 * query ranges when each range is embedded in a full-length partial whose
 * other rows are empty).  Per row r:
 *
 *     L = ln sum_p exp(lses[p][r]),   out[r,:] = sum_p exp(lses[p][r] - L) * partials[p][r,:]
 *
 * A partial row with lse = -inf has weight 0 and its values are never used
 * (they may be NaN or uninitialised); if every partial is empty the row gets
 * out = 0, lse_out = -inf.
 *
 * partials, lses: HOST arrays of n device pointers ([rows,d] and [rows] fp32);
 * they are read during the call only.  out [rows,d] may alias one of the
 * partials; lse_out [rows] is optional (NULL to skip) and must not alias any
 * of the lses.  1 <= n <= PDA_MAX_PARTIALS; d % 4 == 0, d <= 256; rows == 0 is a no-op.
 */
int pda_attn_merge(const float* const* partials, const float* const* lses, int n,
                   float* out, float* lse_out, int64_t rows, int d, void* stream);

/*
 * PipeSP's head-chunk pipeline (Algorithm 1, steps 2-9) on one GPU's share of
 * heads.  Heads are issued in order in groups of heads_per_group (the last
 * group may be smaller; the paper uses one head per step).  For group g:
 *
 *   compute stream: attention over the group's heads  (step 3)
 *   record event g on the compute stream              (step 5)
 *   drain stream waits for event g                    (step 6)
 *   drain stream: hand-off of the group's result      (step 7; stands in for the
 *                 All-to-All, which needs more than one GPU: the group's slice
 *                 of out is copied to the same slice of sink)
 *
 * so the hand-off of group g overlaps the attention of group g+1.  out/lse of
 * group g are what one pda_attn_fwd call over the group's heads writes (a call
 * over all heads agrees up to the rounding of probabilities: which query tiles
 * are computed as merged key-range partials depends on the launch size).
 *
 * sink: optional device [B,H,Sq,d] fp32, not overlapping out (NULL: the drain stream only waits).
 * group_ms: optional HOST array of ceil(H/heads_per_group) floats receiving the
 * compute-stream time of each group; total_ms: optional HOST float receiving
 * the time from the first launch to the end of the last hand-off.  If either
 * is non-NULL the call synchronises both streams before returning; otherwise
 * it returns after enqueueing and the caller must wait on BOTH streams.
 * The two streams must differ.  Events are created and destroyed inside the call.
 * The untimed form may be captured into a HIP graph once the compute stream has run an
 * attention launch outside the capture (its workspace exists then): begin the capture on the
 * compute stream, call, make the compute stream wait for the drain stream, end the capture.
 */
int pda_headchunk_run(const void* q, const void* k, const void* v, float* out, float* lse,
                      int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                      int64_t kv_valid_len, int heads_per_group,
                      void* compute_stream, void* drain_stream,
                      float* sink, float* group_ms, float* total_ms);

/* ---- steps next to the attention call ------------------------------------------------------ */

#define PDA_MAX_LOCAL_HEADS 64

/* Layouts of the hand-off target of pda_headchunk_run_ex. */
#define PDA_SINK_HEAD_MAJOR    0  /* [B,H,Sq,d], as out (what pda_headchunk_run does) */
#define PDA_SINK_TOKEN_ARRIVAL 1  /* [B,Sq,H,d], heads in the order PipeSP's per-head exchanges deliver them */
#define PDA_SINK_TOKEN_FINAL   2  /* [B,Sq,H,d], heads in the original order: post-processing folded into the hand-off */

/*
 * PipeSP post-processing, Algorithm 1 steps 10-13, as one pass over the data:
 * concat(chunks, dim=1) -> view(-1,h,n,D) -> permute(0,2,1,3) -> view(-1,h*n,D), i.e. the map
 * Psi of the Supplement's consistency proof,
 *
 *     hidden[r, i*h + j, :] = chunks[j][r, i, :]      r < rows, i < n, j < h
 *
 * chunks: HOST array of h device pointers.  chunks[j] is what the exchange of pipeline step j
 * delivered: [rows, n, D] fp32, one piece per source GPU i, rows = flattened (batch, local token).
 * chunk_row_stride is the distance in floats between consecutive rows of a chunk: n*D for
 * separate compact chunks, h*n*D when the chunks are the slices t_mod + j*n*D of one already
 * concatenated [rows, h*n, D] tensor (head order k_mod = j*n + i).  hidden: device [rows, n*h, D]
 * (head order k_orig = i*h + j); must not overlap any chunk.
 * 1 <= h <= PDA_MAX_LOCAL_HEADS, n >= 1, D % 4 == 0, chunk_row_stride % 4 == 0 and >= n*D,
 * 16-byte aligned pointers; rows == 0 is a no-op.
 */
int pda_pipesp_postprocess(const float* const* chunks, int h, int n, int64_t chunk_row_stride,
                           float* hidden, int64_t rows, int D, void* stream);

/*
 * pda_headchunk_run with an explicit list of head groups and a choice of hand-off layout.
 *
 * group_sizes: HOST array of n_groups positive counts summing to H; group g covers the next
 * group_sizes[g] heads (unequal groups: a head count that does not divide over the GPUs, Attention
 * Co-processing section, last paragraph of the performance analysis).
 *
 * sink_layout / sp_ranks: with PDA_SINK_HEAD_MAJOR the hand-off is pda_headchunk_run's.  The two
 * token-major layouts model the receive side of PipeSP's exchange for n = sp_ranks simulated
 * GPUs on one device: H = n*h, global head k = i*h + j is local head j of GPU i, and the hand-off
 * of a group writes each of its heads into sink[b, s, slot, :] with slot = j*n + i
 * (PDA_SINK_TOKEN_ARRIVAL: the interleaved order that Algorithm 1 step 10 produces, to be fixed
 * by pda_pipesp_postprocess with rows = B*Sq) or slot = i*h + j (PDA_SINK_TOKEN_FINAL: steps
 * 11-13 folded into the copy).  They need sink != NULL and H % sp_ranks == 0; sp_ranks >= 1.
 * Everything else as pda_headchunk_run; group_ms has n_groups entries.
 */
int pda_headchunk_run_ex(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, const int* group_sizes, int n_groups,
                         int sp_ranks, int sink_layout,
                         void* compute_stream, void* drain_stream,
                         float* sink, float* group_ms, float* total_ms);

/*
 * Pre-attention pack: token-major fp32 projections x [B,S,H,d] (one row of H*d features per
 * token) to the head-major bf16 tensor y [B,H,S,d] that Algorithm 1 slices per head.  With
 * unit_rms != 0 every d-vector is first divided by its own root mean square (fp32 arithmetic;
 * a zero vector stays zero).  Every element is multiplied by premul (finite; 1 for none) before
 * the one rounding to bf16 (nearest even): a Q packed with premul = scale * log2(e) goes with
 * pda_attn_fwd_base2.  d must be 64 or 128; x and y 16-byte aligned and distinct; B*S*H == 0 is
 * a no-op.
 */
int pda_pack_heads(const float* x, void* y, int B, int64_t S, int H, int d, int unit_rms, float premul, void* stream);

/*
 * Planner formulas (host only; every pointer below is a HOST pointer; no device work).
 *
 * pda_plan_n_decode: "Optimal GPU partitioning" of the Diffusion-VAE decoupling,
 *     N_decode = ceil( T_decode / (T_decode + T_denoise) * N ),
 * evaluated in double precision in that order and clamped to [1, N-1] (both groups need a GPU).
 * Needs N >= 2 and positive finite times.
 *
 * pda_plan_aco: Attention Co-processing, performance analysis (Eq. 1-3),
 *     T_baseline = t_L + t_A,  T_coop = t_L + t_A * N_denoise / (N_denoise + N_decode),
 *     S = T_baseline / T_coop.
 * Needs n_denoise >= 1, n_decode >= 0, t_L, t_A >= 0 and finite, t_L + t_A > 0.  Any output may be NULL.
 *
 * pda_plan_head_padding: heads padded to a multiple of the GPU count (same section):
 * padded = ceil(H/n)*n, per GPU = padded/n, GPUs effectively needed = ceil(H / per GPU)
 * (H = 24, n = 7 gives 28, 4, 6).  pda_plan_ragged_groups: the split without padding, group i
 * gets floor(H/n) heads plus one if i < H mod n; group_sizes has n entries (zeros if H < n).
 */
int pda_plan_n_decode(double t_denoise, double t_decode, int N, int* n_decode);
int pda_plan_aco(double t_L, double t_A, int n_denoise, int n_decode,
                 double* t_baseline, double* t_coop, double* speedup);
int pda_plan_head_padding(int H, int n_denoise, int* padded_heads, int* heads_per_gpu, int* gpus_needed);
int pda_plan_ragged_groups(int H, int n, int* group_sizes);

/*
 * Measurement aid for the roofline: the rate the matrix cores alone sustain on this device on
 * the caller's data.  Runs a loop of nothing but bf16 MFMAs (32x32x16, fp32 accumulate, the
 * instruction the attention kernel uses) whose operand fragments are read once from
 * operands (device, bf16, n_elems >= 4096 elements, 16-byte aligned; e.g. the Q tensor of the
 * workload), on every compute unit with two wavefronts per SIMD, for mfma_per_wave MFMAs per
 * wavefront (rounded up to a multiple of 8; about 1e6 gives a 30 ms run), timed with events on
 * the stream.  SYNCHRONOUS.  tflops (HOST pointer) receives the measured rate in TFLOP/s,
 * ms (HOST, optional) the duration.  The sustained clock, and with it this rate, depends on the
 * operand values (constant operands run faster than random ones).
 */
int pda_probe_mfma_rate(const void* operands, int64_t n_elems, int64_t mfma_per_wave,
                        float* tflops, float* ms, void* stream);

/*
 * pda_probe_mfma_rate with the other instruction classes of the attention kernel's inner loop
 * added to the MFMA loop at the kernel's own density, so that what each class costs under the
 * chip's power limit can be measured on the caller's data, one class after the other:
 *   mix 0: MFMAs only (pda_probe_mfma_rate)
 *   mix 1: + the softmax arithmetic: per MFMA one fp32 multiply-add, one exponential, one add
 *          and half a conversion to bf16
 *   mix 2: + the MFMA operand fragments read from LDS as the kernel reads them: per two MFMAs
 *          one 16-byte read and one pair of transposing 8-byte reads per lane
 *   mix 3: mix 2 with half the reads (what a wavefront owning 64 instead of 32 query rows needs)
 * No global->LDS copies, no barriers, no dependencies between the classes: an upper bound for the
 * kernel's steady state.  Arguments and conventions as pda_probe_mfma_rate; SYNCHRONOUS.
 */
int pda_probe_loop_rate(const void* operands, int64_t n_elems, int64_t mfma_per_wave, int mix,
                        float* tflops, float* ms, void* stream);

/* Message of the calling thread's most recent failure ("" if none). Never NULL. */
const char* pda_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int pda_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPEDIT_ATTN_H */
