// C ABI of libpipedit_attn: argument validation, launches, and the head-chunk scheduler.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdarg>
#include <atomic>
#include <cstdio>
#include <map>
#include <mutex>
#include <utility>
#include <vector>
#include "../../include/pipedit_attn.h"
#include "attn_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(PDA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shared validation of the attention shape arguments.  Returns PDA_OK or an error code.
int check_attn_args(const void* q, const void* k, const void* v, const float* out, const float* lse,
                    int B, int H, int64_t Sq, int64_t Skv, int d, float scale, int64_t kv_valid_len) {
    if (B < 0 || H < 0 || Sq < 0 || Skv < 0) return fail(PDA_ERR_INVALID_ARG, "negative size (B=%d H=%d Sq=%lld Skv=%lld)", B, H, (long long)Sq, (long long)Skv);
    if (d != 64 && d != 128) return fail(PDA_ERR_UNSUPPORTED, "head dim d=%d not supported (64 or 128)", d);
    if (kv_valid_len < 0 || kv_valid_len > Skv) return fail(PDA_ERR_INVALID_ARG, "kv_valid_len=%lld outside [0, Skv=%lld]", (long long)kv_valid_len, (long long)Skv);
    if (!(scale >= 0.0f) || !std::isfinite(scale)) return fail(PDA_ERR_INVALID_ARG, "scale must be finite and >= 0");
    if (Sq > (int64_t)1 << 31 || Skv >= (int64_t)1 << 31) return fail(PDA_ERR_UNSUPPORTED, "sequence length beyond 2^31");
    if ((double)B * H * (double)(Sq > Skv ? Sq : Skv) * d >= 1099511627776.0) return fail(PDA_ERR_UNSUPPORTED, "B*H*S*d overflows 2^40 elements");
    if ((int64_t)B * H > 65535) return fail(PDA_ERR_UNSUPPORTED, "B*H > 65535");
    const bool empty = (B == 0 || H == 0 || Sq == 0);
    if (!empty) {
        if (!q || !out || !lse) return fail(PDA_ERR_INVALID_ARG, "null q/out/lse");
        if (kv_valid_len > 0 && (!k || !v)) return fail(PDA_ERR_INVALID_ARG, "null k/v");
        if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return fail(PDA_ERR_UNSUPPORTED, "q/k/v/out must be 16-byte aligned");
        if (reinterpret_cast<uintptr_t>(lse) & 3u) return fail(PDA_ERR_UNSUPPORTED, "lse must be 4-byte aligned");
    }
    return PDA_OK;
}

// Batch and head strides (elements) of the four tensor kinds of an attention call.
struct Strides {
    int64_t q_bs, q_hs, kv_bs, kv_hs, o_bs, o_hs, l_bs, l_hs;
};

Strides compact_strides(int H, int64_t Sq, int64_t Skv, int d) {
    return {(int64_t)H * Sq * d, Sq * d, (int64_t)H * Skv * d, Skv * d, (int64_t)H * Sq * d, Sq * d, (int64_t)H * Sq, Sq};
}

// Launch attention for hg heads of B batches; the pointers address the first of those heads.
// base2: the scores q.k are already in log2 units (scale is then ln 2 and is not applied again).
hipError_t launch_strided(const void* q, const void* k, const void* v, float* out, float* lse,
                          int B, int hg, int64_t Sq, int d, const Strides& s, float scale, int64_t n_v, hipStream_t st,
                          int variant, bool base2, bool out_bf16, float* ws, int64_t ws_slots) {
    pda::AttnParams p{};
    p.q = static_cast<const __bf16*>(q);
    p.k = static_cast<const __bf16*>(k);
    p.v = static_cast<const __bf16*>(v);
    p.out = out;
    p.lse = lse;
    p.Sq = Sq;
    p.n_v = n_v;
    p.q_hs = s.q_hs;   p.q_bs = s.q_bs;
    p.kv_hs = s.kv_hs; p.kv_bs = s.kv_bs;
    p.o_hs = s.o_hs;   p.o_bs = s.o_bs;
    p.l_hs = s.l_hs;   p.l_bs = s.l_bs;
    p.Hg = hg;
    p.scale = scale;
    // scale 0 is run with a tiny positive factor so that hidden keys (-inf scores) still get exp2(-inf) = 0
    p.scale_log2e = base2 ? 1.0f : std::fmax(scale * 1.4426950408889634f, 1e-37f);
    p.base2 = base2 ? 1 : 0;
    p.out_bf16 = out_bf16 ? 1 : 0;
    return pda::launch_attn_fwd(p, B * hg, d, variant, ws, ws_slots, st);
}

}  // namespace

namespace pda {

hipError_t device_cu_count(int* n_cu) {
    static std::atomic<int> cu[KernelSetup::MAX_DEV] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool cached = dev >= 0 && dev < KernelSetup::MAX_DEV;
    int v = cached ? cu[dev].load(std::memory_order_acquire) : 0;
    if (v == 0) {
        if ((e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        if (cached) cu[dev].store(v, std::memory_order_release);
    }
    *n_cu = v;
    return hipSuccess;
}

}  // namespace pda

namespace {

// ---- workspaces of the software-pipelined kernel: key-range partials and the work counters ------
//
// (1) Cached: one buffer per (device, stream), allocated (and its counters zeroed) the first time
// the kernel is launched on that stream, with the largest size any launch can need on the device
// (a function of its CU count alone), so it never grows, is never freed and the launch path never
// synchronises after that.  Launches on one stream are ordered and share it.
struct CachedWs { float* ptr; int64_t slots; };
int cached_workspace(hipStream_t st, int64_t need_slots, CachedWs* out) {
    static std::mutex mu;
    static std::map<std::pair<int, hipStream_t>, CachedWs> pool;
    int dev = 0, n_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = pda::device_cu_count(&n_cu);
    if (e != hipSuccess) return hip_fail(e, "device query");
    std::lock_guard<std::mutex> lock(mu);
    CachedWs& w = pool[{dev, st}];
    if (!w.ptr) {
        const int64_t slots = pda::max_tail_slots(n_cu, true);
        void* ptr = nullptr;
        const size_t bytes = ((size_t)slots * pda::kSlotFloats + pda::kCounterFloats) * sizeof(float);
        e = hipMalloc(&ptr, bytes);
        if (e == hipErrorOutOfMemory) {
            (void)hipGetLastError();
            return fail(PDA_ERR_NOMEM, "no device memory for the %lld MB workspace of this stream", (long long)(bytes >> 20));
        }
        if (e != hipSuccess) return hip_fail(e, "workspace allocation");
        // the work counters start at zero (every launch leaves them at zero again); part of this one-time set-up
        e = hipMemset(static_cast<float*>(ptr) + (size_t)slots * pda::kSlotFloats, 0, pda::kCounterFloats * sizeof(float));
        if (e != hipSuccess) { (void)hipFree(ptr); return hip_fail(e, "workspace set-up"); }
        w.ptr = static_cast<float*>(ptr);
        w.slots = slots;
    }
    if (need_slots > w.slots) return fail(PDA_ERR_UNSUPPORTED, "launch needs %lld workspace slots, the stream's buffer has %lld", (long long)need_slots, (long long)w.slots);
    *out = w;
    return PDA_OK;
}

// (2) Static: for callers that cannot allocate (pda_attn_fwd_noalloc).  A file-scope device array;
// every GPU the library runs on holds its own copy at its own address, looked up once per device.
// In host code the array's NAME is not a device address: only the pointer hipGetSymbolAddress
// returns is ever handed to a kernel.
constexpr int64_t kStaticSlots = PDA_NOALLOC_MAX_SLOTS;
static __device__ __align__(256) float scratch[kStaticSlots * pda::kSlotFloats + pda::kCounterFloats];   // zero-initialised
static_assert(sizeof(scratch) == PDA_NOALLOC_SCRATCH_BYTES, "header and library disagree");

int static_workspace(float** out) {
    static std::mutex mu;
    static float* per_dev[pda::KernelSetup::MAX_DEV] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "device query");
    if (dev < 0 || dev >= pda::KernelSetup::MAX_DEV) return fail(PDA_ERR_UNSUPPORTED, "device index %d beyond %d", dev, pda::KernelSetup::MAX_DEV);
    std::lock_guard<std::mutex> lock(mu);
    if (!per_dev[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return fail(PDA_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
        per_dev[dev] = static_cast<float*>(ptr);
    }
    *out = per_dev[dev];
    return PDA_OK;
}

enum WsKind { WS_CACHED, WS_STATIC };

// Validated attention launch for hg heads of B batches with the workspace the launch needs.
int launch_checked(const void* q, const void* k, const void* v, float* out, float* lse,
                   int B, int hg, int64_t Sq, int d, const Strides& s, float scale, int64_t n_v, hipStream_t st,
                   int variant, bool base2, bool out_bf16, WsKind kind) {
    float* ws = nullptr;
    int64_t ws_slots = 0;
    if (out_bf16 && variant != 3) variant = 0;           // only the software-pipelined kernel writes bf16
    if (pda::uses_sp_kernel(d, variant, n_v)) {
        int n_cu = 0;
        hipError_t e = pda::device_cu_count(&n_cu);
        if (e != hipSuccess) return hip_fail(e, "device query");
        // every launch of this kernel uses a workspace: its work counters, and the partial slots of cut tiles
        const int64_t need = pda::tail_slots(pda::plan_tail(Sq, B * hg, n_v, n_cu), out_bf16);
        if (kind == WS_STATIC) {
            if (need > kStaticSlots)
                return fail(PDA_ERR_UNSUPPORTED, "this launch needs %lld partial slots (%lld bytes) of scratch; the static buffer holds %lld (%lld bytes)",
                            (long long)need, (long long)(need * pda::kSlotFloats * sizeof(float)),
                            (long long)kStaticSlots, (long long)PDA_NOALLOC_SCRATCH_BYTES);
            int rc = static_workspace(&ws);
            if (rc != PDA_OK) return rc;
            ws_slots = kStaticSlots;
        } else {
            CachedWs w{};
            int rc = cached_workspace(st, need, &w);
            if (rc != PDA_OK) return rc;
            ws = w.ptr;
            ws_slots = w.slots;
        }
    }
    hipError_t e = launch_strided(q, k, v, out, lse, B, hg, Sq, d, s, scale, n_v, st, variant, base2, out_bf16, ws, ws_slots);
    if (e != hipSuccess) return hip_fail(e, "attention launch");
    return PDA_OK;
}

}  // namespace

namespace {

// Launch attention for heads [h0, h0+hg) of compact [B,H,S,d] tensors.  Returns a pda_status.
int launch_heads(const void* q, const void* k, const void* v, float* out, float* lse,
                 int B, int H, int64_t Sq, int64_t Skv, int d, float scale, int64_t n_v,
                 int h0, int hg, hipStream_t st, int variant = 0, WsKind kind = WS_CACHED) {
    return launch_checked(static_cast<const __bf16*>(q) + (int64_t)h0 * Sq * d,
                          static_cast<const __bf16*>(k) + (int64_t)h0 * Skv * d,
                          static_cast<const __bf16*>(v) + (int64_t)h0 * Skv * d,
                          out + (int64_t)h0 * Sq * d, lse + (int64_t)h0 * Sq,
                          B, hg, Sq, d, compact_strides(H, Sq, Skv, d), scale, n_v, st, variant, false, false, kind);
}

// The head-chunk pipeline (Algorithm 1, steps 2-9) over the given groups; arguments already validated.
int run_pipeline(const void* q, const void* k, const void* v, float* out, float* lse,
                 int B, int H, int64_t Sq, int64_t Skv, int d, float scale, int64_t kv_valid_len,
                 const std::vector<int>& sizes, int sp_ranks, int sink_layout,
                 void* compute_stream, void* drain_stream, float* sink, float* group_ms, float* total_ms) {
    if (compute_stream == drain_stream) return fail(PDA_ERR_INVALID_ARG, "compute and drain streams must differ");
    if (sink && !aligned16(sink)) return fail(PDA_ERR_UNSUPPORTED, "sink must be 16-byte aligned");
    if (sink) {
        const char* o0 = reinterpret_cast<const char*>(out);
        const char* s0 = reinterpret_cast<const char*>(sink);
        const size_t bytes = (size_t)B * H * Sq * d * sizeof(float);
        if (o0 < s0 + bytes && s0 < o0 + bytes) return fail(PDA_ERR_INVALID_ARG, "sink must not overlap out");
    }
    const int n_groups = (int)sizes.size();
    if (B == 0 || H == 0 || Sq == 0) {
        if (total_ms) *total_ms = 0.f;
        for (int g = 0; group_ms && g < n_groups; ++g) group_ms[g] = 0.f;
        return PDA_OK;
    }
    hipStream_t cs = static_cast<hipStream_t>(compute_stream), ds = static_cast<hipStream_t>(drain_stream);
    const bool timed = group_ms != nullptr || total_ms != nullptr;

    // Events: done[g] orders the hand-off of group g after its attention (Algorithm 1, steps 5-6);
    // beg[g]/done[g] also time the group when timing is requested.
    std::vector<hipEvent_t> done(n_groups, nullptr), beg(timed ? n_groups : 0, nullptr);
    hipEvent_t drain_end = nullptr;
    hipError_t e = hipSuccess;
    const unsigned flags = timed ? hipEventDefault : hipEventDisableTiming;
    auto cleanup = [&]() {
        for (auto ev : done) if (ev) (void)hipEventDestroy(ev);
        for (auto ev : beg) if (ev) (void)hipEventDestroy(ev);
        if (drain_end) (void)hipEventDestroy(drain_end);
    };
    for (int g = 0; g < n_groups && e == hipSuccess; ++g) {
        e = hipEventCreateWithFlags(&done[g], flags);
        if (e == hipSuccess && timed) e = hipEventCreateWithFlags(&beg[g], hipEventDefault);
    }
    if (e == hipSuccess && timed) e = hipEventCreateWithFlags(&drain_end, hipEventDefault);
    if (e != hipSuccess) { cleanup(); return hip_fail(e, "event creation"); }

    const int h_local = H / sp_ranks;
    int rc = PDA_OK;
    for (int g = 0, h0 = 0; g < n_groups; h0 += sizes[g], ++g) {
        const int hg = sizes[g];
        if (timed && (e = hipEventRecord(beg[g], cs)) != hipSuccess) break;
        if ((rc = launch_heads(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, h0, hg, cs)) != PDA_OK) break;
        if ((e = hipEventRecord(done[g], cs)) != hipSuccess) break;
        if ((e = hipStreamWaitEvent(ds, done[g], 0)) != hipSuccess) break;
        if (sink) {
            // hand-off of this group's result (step 7): its slice of out goes to the same slice of
            // sink, or into the token-major buffer at the head slots the layout asks for
            for (int b = 0; b < B && e == hipSuccess; ++b) {
                const int64_t off = ((int64_t)b * H + h0) * Sq * d;
                if (sink_layout == PDA_SINK_HEAD_MAJOR)
                    e = pda::launch_copy_f32(out + off, sink + off, (int64_t)hg * Sq * d, ds);
                else
                    e = pda::launch_scatter_heads(out + off, sink + (int64_t)b * Sq * H * d, Sq, d, hg, H, h0, h_local,
                                                  sp_ranks, sink_layout == PDA_SINK_TOKEN_ARRIVAL, ds);
            }
            if (e != hipSuccess) break;
        }
    }
    if (rc == PDA_OK && e == hipSuccess && timed) e = hipEventRecord(drain_end, ds);
    if (rc != PDA_OK || e != hipSuccess) {
        (void)hipStreamSynchronize(cs);
        (void)hipStreamSynchronize(ds);
        cleanup();
        return rc != PDA_OK ? rc : hip_fail(e, "head-chunk pipeline");   // rc: the message is already set
    }
    if (timed) {
        if ((e = hipStreamSynchronize(cs)) == hipSuccess) e = hipStreamSynchronize(ds);
        float ms = 0.f;
        for (int g = 0; g < n_groups && e == hipSuccess; ++g) {
            e = hipEventElapsedTime(&ms, beg[g], done[g]);
            if (group_ms) group_ms[g] = ms;
        }
        if (e == hipSuccess && total_ms) {
            e = hipEventElapsedTime(&ms, beg[0], drain_end);
            *total_ms = ms;
        }
        cleanup();
        if (e != hipSuccess) return hip_fail(e, "head-chunk timing");
        return PDA_OK;
    }
    // Untimed: destroying a recorded event is allowed; its resources are released once it completes.
    cleanup();
    return PDA_OK;
}

}  // namespace

extern "C" {

const char* pda_last_error(void) { return g_err; }

int pda_version(void) { return 310; }

int pda_attn_fwd(const void* q, const void* k, const void* v, float* out, float* lse,
                 int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                 int64_t kv_valid_len, int64_t q_offset, void* stream) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (q_offset < 0) return fail(PDA_ERR_INVALID_ARG, "q_offset=%lld is negative", (long long)q_offset);
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    return launch_heads(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, 0, H, static_cast<hipStream_t>(stream));
}

int pda_attn_fwd_noalloc(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, int64_t q_offset, void* stream) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (q_offset < 0) return fail(PDA_ERR_INVALID_ARG, "q_offset=%lld is negative", (long long)q_offset);
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    return launch_heads(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, 0, H, static_cast<hipStream_t>(stream),
                        0, WS_STATIC);
}

int pda_attn_fwd_variant(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, int variant, void* stream) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (variant < 0 || variant > 3) return fail(PDA_ERR_INVALID_ARG, "variant=%d (0..3)", variant);
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    return launch_heads(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, 0, H, static_cast<hipStream_t>(stream), variant);
}

int pda_attn_tail_plan(int B, int H, int64_t Sq, int64_t kv_valid_len, int d, int n_cu,
                       int64_t* n_tiles, int64_t* n_cut, int* split, int64_t* part_offsets, int64_t* workspace_slots) {
    if (B < 0 || H < 0 || Sq < 0 || kv_valid_len < 0) return fail(PDA_ERR_INVALID_ARG, "negative size");
    if (d != 64 && d != 128) return fail(PDA_ERR_UNSUPPORTED, "head dim d=%d not supported (64 or 128)", d);
    if ((int64_t)B * H > 65535) return fail(PDA_ERR_UNSUPPORTED, "B*H > 65535");
    if (n_cu < 0) return fail(PDA_ERR_INVALID_ARG, "n_cu=%d is negative", n_cu);
    if (n_cu == 0) {
        hipError_t e = pda::device_cu_count(&n_cu);
        if (e != hipSuccess) return hip_fail(e, "device query");
    }
    pda::TailPlan t{};
    t.split = 1;
    if (pda::uses_sp_kernel(d, 0, kv_valid_len) && (int64_t)B * H * Sq > 0) t = pda::plan_tail(Sq, B * H, kv_valid_len, n_cu);
    if (n_tiles) *n_tiles = t.n_tiles;
    if (n_cut) *n_cut = t.n_cut;
    if (split) *split = t.split;
    if (part_offsets)
        for (int j = 0; j <= PDA_MAX_KEY_RANGES; ++j) part_offsets[j] = t.split > 1 ? t.part_off[j] : (j == 0 ? 0 : kv_valid_len);
    if (workspace_slots) *workspace_slots = pda::tail_slots(t, false);
    return PDA_OK;
}

int pda_attn_fwd_bf16out(const void* q, const void* k, const void* v, void* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, void* stream) {
    int rc = check_attn_args(q, k, v, static_cast<const float*>(out), lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    return launch_checked(q, k, v, static_cast<float*>(out), lse, B, H, Sq, d, compact_strides(H, Sq, Skv, d),
                          scale, kv_valid_len, static_cast<hipStream_t>(stream), 0, false, true, WS_CACHED);
}

int pda_attn_fwd_base2(const void* q, const void* k, const void* v, float* out, float* lse,
                       int B, int H, int64_t Sq, int64_t Skv, int d, int64_t kv_valid_len, void* stream) {
    const float ln2 = 0.6931471805599453f;
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, ln2, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    return launch_checked(q, k, v, out, lse, B, H, Sq, d, compact_strides(H, Sq, Skv, d), ln2, kv_valid_len,
                          static_cast<hipStream_t>(stream), 0, true, false, WS_CACHED);
}

int pda_attn_fwd_strided(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d,
                         int64_t q_batch_stride, int64_t q_head_stride,
                         int64_t kv_batch_stride, int64_t kv_head_stride,
                         int64_t out_batch_stride, int64_t out_head_stride,
                         int64_t lse_batch_stride, int64_t lse_head_stride,
                         float scale, int64_t kv_valid_len, int64_t q_offset, void* stream) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (q_offset < 0) return fail(PDA_ERR_INVALID_ARG, "q_offset=%lld is negative", (long long)q_offset);
    const Strides s{q_batch_stride, q_head_stride, kv_batch_stride, kv_head_stride,
                    out_batch_stride, out_head_stride, lse_batch_stride, lse_head_stride};
    const int64_t all[8] = {s.q_bs, s.q_hs, s.kv_bs, s.kv_hs, s.o_bs, s.o_hs, s.l_bs, s.l_hs};
    for (int64_t x : all)
        if (x < 0 || x >= ((int64_t)1 << 40)) return fail(PDA_ERR_INVALID_ARG, "stride %lld outside [0, 2^40)", (long long)x);
    if ((s.q_bs | s.q_hs | s.kv_bs | s.kv_hs) % 8 != 0) return fail(PDA_ERR_UNSUPPORTED, "q and k/v strides must be multiples of 8 elements");
    if ((s.o_bs | s.o_hs) % 4 != 0) return fail(PDA_ERR_UNSUPPORTED, "out strides must be multiples of 4 elements");
    if (H > 1 && (s.o_hs < Sq * d || s.l_hs < Sq)) return fail(PDA_ERR_INVALID_ARG, "heads of out/lse overlap (head stride too small)");
    if (B > 1 && (s.o_bs < (int64_t)(H - 1) * s.o_hs + Sq * d || s.l_bs < (int64_t)(H - 1) * s.l_hs + Sq))
        return fail(PDA_ERR_INVALID_ARG, "batches of out/lse overlap (batch stride too small)");
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    return launch_checked(q, k, v, out, lse, B, H, Sq, d, s, scale, kv_valid_len, static_cast<hipStream_t>(stream),
                          0, false, false, WS_CACHED);
}

int pda_attn_merge(const float* const* partials, const float* const* lses, int n,
                   float* out, float* lse_out, int64_t rows, int d, void* stream) {
    if (n < 1) return fail(PDA_ERR_INVALID_ARG, "n=%d partials (need >= 1)", n);
    if (n > PDA_MAX_PARTIALS) return fail(PDA_ERR_UNSUPPORTED, "n=%d exceeds PDA_MAX_PARTIALS=%d", n, PDA_MAX_PARTIALS);
    if (rows < 0) return fail(PDA_ERR_INVALID_ARG, "rows=%lld is negative", (long long)rows);
    if (d < 4 || d > 256 || d % 4 != 0) return fail(PDA_ERR_UNSUPPORTED, "d=%d (need a multiple of 4 in [4,256])", d);
    if (!partials || !lses) return fail(PDA_ERR_INVALID_ARG, "null pointer array");
    if ((double)rows * d >= 1099511627776.0) return fail(PDA_ERR_UNSUPPORTED, "rows*d overflows 2^40 elements");
    if (rows == 0) return PDA_OK;
    if (!out) return fail(PDA_ERR_INVALID_ARG, "null out");
    if (!aligned16(out)) return fail(PDA_ERR_UNSUPPORTED, "out must be 16-byte aligned");
    pda::MergeParams p;
    for (int j = 0; j < n; ++j) {
        if (!partials[j] || !lses[j]) return fail(PDA_ERR_INVALID_ARG, "null partial or lse at index %d", j);
        if (!aligned16(partials[j])) return fail(PDA_ERR_UNSUPPORTED, "partial %d must be 16-byte aligned", j);
        if (lse_out && lse_out == lses[j]) return fail(PDA_ERR_INVALID_ARG, "lse_out must not alias lses[%d]", j);
        p.part[j] = partials[j];
        p.lse[j] = lses[j];
    }
    for (int j = n; j < 16; ++j) { p.part[j] = nullptr; p.lse[j] = nullptr; }
    p.out = out;
    p.lse_out = lse_out;
    p.rows = rows;
    p.n = n;
    hipError_t e = pda::launch_merge(p, d, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "merge launch");
    return PDA_OK;
}

int pda_headchunk_run(const void* q, const void* k, const void* v, float* out, float* lse,
                      int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                      int64_t kv_valid_len, int heads_per_group,
                      void* compute_stream, void* drain_stream,
                      float* sink, float* group_ms, float* total_ms) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (heads_per_group < 1) return fail(PDA_ERR_INVALID_ARG, "heads_per_group=%d (need >= 1)", heads_per_group);
    std::vector<int> sizes;
    for (int h0 = 0; h0 < H; h0 += heads_per_group) sizes.push_back(h0 + heads_per_group <= H ? heads_per_group : H - h0);
    return run_pipeline(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, sizes, 1, PDA_SINK_HEAD_MAJOR,
                        compute_stream, drain_stream, sink, group_ms, total_ms);
}

int pda_headchunk_run_ex(const void* q, const void* k, const void* v, float* out, float* lse,
                         int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                         int64_t kv_valid_len, const int* group_sizes, int n_groups,
                         int sp_ranks, int sink_layout,
                         void* compute_stream, void* drain_stream,
                         float* sink, float* group_ms, float* total_ms) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (n_groups < 0 || (n_groups > 0 && !group_sizes)) return fail(PDA_ERR_INVALID_ARG, "bad group list (n_groups=%d)", n_groups);
    int64_t sum = 0;
    for (int g = 0; g < n_groups; ++g) {
        if (group_sizes[g] < 1) return fail(PDA_ERR_INVALID_ARG, "group_sizes[%d]=%d (need >= 1)", g, group_sizes[g]);
        sum += group_sizes[g];
    }
    if (sum != H) return fail(PDA_ERR_INVALID_ARG, "group sizes sum to %lld, H=%d", (long long)sum, H);
    if (sink_layout != PDA_SINK_HEAD_MAJOR && sink_layout != PDA_SINK_TOKEN_ARRIVAL && sink_layout != PDA_SINK_TOKEN_FINAL)
        return fail(PDA_ERR_INVALID_ARG, "unknown sink_layout=%d", sink_layout);
    if (sp_ranks < 1) return fail(PDA_ERR_INVALID_ARG, "sp_ranks=%d (need >= 1)", sp_ranks);
    if (sink_layout != PDA_SINK_HEAD_MAJOR) {
        if (!sink) return fail(PDA_ERR_INVALID_ARG, "a token-major hand-off needs a sink");
        if (H % sp_ranks != 0) return fail(PDA_ERR_INVALID_ARG, "H=%d is not a multiple of sp_ranks=%d", H, sp_ranks);
    }
    return run_pipeline(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len,
                        std::vector<int>(group_sizes, group_sizes + n_groups), sp_ranks, sink_layout,
                        compute_stream, drain_stream, sink, group_ms, total_ms);
}

int pda_pipesp_postprocess(const float* const* chunks, int h, int n, int64_t chunk_row_stride,
                           float* hidden, int64_t rows, int D, void* stream) {
    if (h < 1 || n < 1) return fail(PDA_ERR_INVALID_ARG, "h=%d n=%d (need >= 1)", h, n);
    if (h > PDA_MAX_LOCAL_HEADS) return fail(PDA_ERR_UNSUPPORTED, "h=%d exceeds PDA_MAX_LOCAL_HEADS=%d", h, PDA_MAX_LOCAL_HEADS);
    if (rows < 0) return fail(PDA_ERR_INVALID_ARG, "rows=%lld is negative", (long long)rows);
    if (D < 4 || D % 4 != 0) return fail(PDA_ERR_UNSUPPORTED, "D=%d (need a positive multiple of 4)", D);
    if ((double)n * D >= 2147483648.0 || (double)n * D * h >= 2147483648.0) return fail(PDA_ERR_UNSUPPORTED, "n*h*D beyond 2^31");
    if (chunk_row_stride < (int64_t)n * D || chunk_row_stride % 4 != 0)
        return fail(PDA_ERR_INVALID_ARG, "chunk_row_stride=%lld (need a multiple of 4, >= n*D=%lld)", (long long)chunk_row_stride, (long long)n * D);
    if ((double)rows * n * h * D >= 1099511627776.0 || (double)rows * (double)chunk_row_stride >= 1099511627776.0)
        return fail(PDA_ERR_UNSUPPORTED, "tensor beyond 2^40 elements");
    if (!chunks) return fail(PDA_ERR_INVALID_ARG, "null chunk array");
    if (rows == 0) return PDA_OK;
    if (!hidden) return fail(PDA_ERR_INVALID_ARG, "null hidden");
    if (!aligned16(hidden)) return fail(PDA_ERR_UNSUPPORTED, "hidden must be 16-byte aligned");
    pda::PostParams p{};
    const char* hid0 = reinterpret_cast<const char*>(hidden);
    const char* hid1 = hid0 + (size_t)rows * n * h * D * sizeof(float);
    for (int j = 0; j < h; ++j) {
        if (!chunks[j]) return fail(PDA_ERR_INVALID_ARG, "null chunk %d", j);
        if (!aligned16(chunks[j])) return fail(PDA_ERR_UNSUPPORTED, "chunk %d must be 16-byte aligned", j);
        const char* c0 = reinterpret_cast<const char*>(chunks[j]);
        const char* c1 = c0 + ((size_t)(rows - 1) * chunk_row_stride + (size_t)n * D) * sizeof(float);
        if (c0 < hid1 && hid0 < c1) return fail(PDA_ERR_INVALID_ARG, "hidden overlaps chunk %d", j);
        p.chunk[j] = chunks[j];
    }
    p.hidden = hidden;
    p.rows = rows;
    p.row_stride4 = chunk_row_stride / 4;
    p.h = h; p.n = n; p.D4 = D / 4;
    hipError_t e = pda::launch_postprocess(p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "post-processing launch");
    return PDA_OK;
}

int pda_pack_heads(const float* x, void* y, int B, int64_t S, int H, int d, int unit_rms, float premul, void* stream) {
    if (B < 0 || H < 0 || S < 0) return fail(PDA_ERR_INVALID_ARG, "negative size (B=%d H=%d S=%lld)", B, H, (long long)S);
    if (d != 64 && d != 128) return fail(PDA_ERR_UNSUPPORTED, "head dim d=%d not supported (64 or 128)", d);
    if ((double)B * H * (double)S * d >= 1099511627776.0) return fail(PDA_ERR_UNSUPPORTED, "B*H*S*d overflows 2^40 elements");
    if (B == 0 || H == 0 || S == 0) return PDA_OK;
    if (!x || !y) return fail(PDA_ERR_INVALID_ARG, "null x/y");
    if (!aligned16(x) || !aligned16(y)) return fail(PDA_ERR_UNSUPPORTED, "x and y must be 16-byte aligned");
    if (static_cast<const void*>(x) == y) return fail(PDA_ERR_INVALID_ARG, "y must not alias x");
    if (!std::isfinite(premul)) return fail(PDA_ERR_INVALID_ARG, "premul must be finite");
    hipError_t e = pda::launch_pack(x, y, B, S, H, d, unit_rms, premul, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "pack launch");
    return PDA_OK;
}

static int probe_rate(const void* operands, int64_t n_elems, int64_t mfma_per_wave, int mix,
                      float* tflops, float* ms, void* stream) {
    if (!operands || !tflops) return fail(PDA_ERR_INVALID_ARG, "null operands/tflops");
    if (n_elems < 4096) return fail(PDA_ERR_INVALID_ARG, "n_elems=%lld (need >= 4096)", (long long)n_elems);
    if (mfma_per_wave < 1 || mfma_per_wave > ((int64_t)1 << 32)) return fail(PDA_ERR_INVALID_ARG, "mfma_per_wave out of range");
    if (mix < 0 || mix > 3) return fail(PDA_ERR_INVALID_ARG, "mix=%d (0..3)", mix);
    if (!aligned16(operands)) return fail(PDA_ERR_UNSUPPORTED, "operands must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    int n_cu = 0;
    hipError_t e = pda::device_cu_count(&n_cu);
    if (e != hipSuccess) return hip_fail(e, "device query");
    CachedWs w{};
    int rc = cached_workspace(st, 1, &w);            // one slot is far more than the 512 floats needed
    if (rc != PDA_OK) return rc;
    float* sink = w.ptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    const int64_t iters = (mfma_per_wave + 15) / 16 * 2;       // units of 8 MFMAs, an even number of them
    float t = 0.f;
    if (e == hipSuccess) e = hipEventRecord(e0, st);
    if (e == hipSuccess) e = pda::launch_mfma_rate(operands, n_elems / 8, iters, n_cu, mix, sink, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(e, "MFMA rate probe");
    const double flop = (double)n_cu * 8.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
    *tflops = (float)(flop / ((double)t * 1e-3) * 1e-12);
    if (ms) *ms = t;
    return PDA_OK;
}

int pda_probe_mfma_rate(const void* operands, int64_t n_elems, int64_t mfma_per_wave,
                        float* tflops, float* ms, void* stream) {
    return probe_rate(operands, n_elems, mfma_per_wave, 0, tflops, ms, stream);
}

int pda_probe_loop_rate(const void* operands, int64_t n_elems, int64_t mfma_per_wave, int mix,
                        float* tflops, float* ms, void* stream) {
    return probe_rate(operands, n_elems, mfma_per_wave, mix, tflops, ms, stream);
}

int pda_plan_n_decode(double t_denoise, double t_decode, int N, int* n_decode) {
    if (!n_decode) return fail(PDA_ERR_INVALID_ARG, "null n_decode");
    if (N < 2) return fail(PDA_ERR_INVALID_ARG, "N=%d (need >= 2: one GPU per group)", N);
    if (!(t_denoise > 0.0) || !(t_decode > 0.0) || !std::isfinite(t_denoise) || !std::isfinite(t_decode))
        return fail(PDA_ERR_INVALID_ARG, "times must be positive and finite");
    const double raw = std::ceil(t_decode / (t_decode + t_denoise) * N);
    int v = (int)raw;
    if (v < 1) v = 1;
    if (v > N - 1) v = N - 1;
    *n_decode = v;
    return PDA_OK;
}

int pda_plan_aco(double t_L, double t_A, int n_denoise, int n_decode,
                 double* t_baseline, double* t_coop, double* speedup) {
    if (n_denoise < 1 || n_decode < 0) return fail(PDA_ERR_INVALID_ARG, "n_denoise=%d n_decode=%d", n_denoise, n_decode);
    if (!(t_L >= 0.0) || !(t_A >= 0.0) || !std::isfinite(t_L) || !std::isfinite(t_A) || !(t_L + t_A > 0.0))
        return fail(PDA_ERR_INVALID_ARG, "times must be finite, >= 0 and not both zero");
    const double base = t_L + t_A;
    const double coop = t_L + t_A * ((double)n_denoise / (double)(n_denoise + n_decode));
    if (t_baseline) *t_baseline = base;
    if (t_coop) *t_coop = coop;
    if (speedup) *speedup = base / coop;
    return PDA_OK;
}

int pda_plan_head_padding(int H, int n_denoise, int* padded_heads, int* heads_per_gpu, int* gpus_needed) {
    if (H < 1 || n_denoise < 1) return fail(PDA_ERR_INVALID_ARG, "H=%d n_denoise=%d (need >= 1)", H, n_denoise);
    const int per = (H + n_denoise - 1) / n_denoise;
    if (padded_heads) *padded_heads = per * n_denoise;
    if (heads_per_gpu) *heads_per_gpu = per;
    if (gpus_needed) *gpus_needed = (H + per - 1) / per;
    return PDA_OK;
}

int pda_plan_ragged_groups(int H, int n, int* group_sizes) {
    if (H < 0 || n < 1) return fail(PDA_ERR_INVALID_ARG, "H=%d n=%d", H, n);
    if (!group_sizes) return fail(PDA_ERR_INVALID_ARG, "null group_sizes");
    for (int i = 0; i < n; ++i) group_sizes[i] = H / n + (i < H % n ? 1 : 0);
    return PDA_OK;
}

}  // extern "C"
