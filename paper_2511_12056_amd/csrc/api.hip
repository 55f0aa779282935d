// C ABI of libpipedit_attn: argument validation, launches, and the head-chunk scheduler.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
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

// Tiling variant of the forward kernel; PDA_ATTN_VARIANT in the environment overrides the default
// (a tuning aid: every variant computes the same function).
int attn_variant() {
    static int v = [] {
        const char* s = getenv("PDA_ATTN_VARIANT");
        return s ? atoi(s) : 0;
    }();
    return v;
}

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

// Launch attention for heads [h0, h0+hg) of compact [B,H,S,d] tensors.
hipError_t launch_heads(const void* q, const void* k, const void* v, float* out, float* lse,
                        int B, int H, int64_t Sq, int64_t Skv, int d, float scale, int64_t n_v,
                        int h0, int hg, hipStream_t st) {
    pda::AttnParams p{};
    p.q = static_cast<const __bf16*>(q) + (int64_t)h0 * Sq * d;
    p.k = static_cast<const __bf16*>(k) + (int64_t)h0 * Skv * d;
    p.v = static_cast<const __bf16*>(v) + (int64_t)h0 * Skv * d;
    p.out = out + (int64_t)h0 * Sq * d;
    p.lse = lse + (int64_t)h0 * Sq;
    p.Sq = Sq;
    p.n_v = n_v;
    p.q_hs = Sq * d;   p.q_bs = (int64_t)H * Sq * d;
    p.kv_hs = Skv * d; p.kv_bs = (int64_t)H * Skv * d;
    p.o_hs = Sq * d;   p.o_bs = (int64_t)H * Sq * d;
    p.l_hs = Sq;       p.l_bs = (int64_t)H * Sq;
    p.Hg = hg;
    p.scale = scale;
    // scale 0 is run with a tiny positive factor so that hidden keys (-inf scores) still get exp2(-inf) = 0
    p.scale_log2e = std::fmax(scale * 1.4426950408889634f, 1e-37f);
    return pda::launch_attn_fwd(p, B * hg, d, attn_variant(), st);
}

}  // namespace

namespace pda {

hipError_t attn_workspace(hipStream_t st, size_t bytes, float** out) {
    struct Buf { void* ptr; size_t size; };
    static std::mutex mu;
    static std::map<std::pair<int, hipStream_t>, Buf> pool;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    Buf& b = pool[{dev, st}];
    if (b.size < bytes) {
        if (b.ptr) {
            // the old buffer may still be read by work queued on this stream
            if ((e = hipStreamSynchronize(st)) != hipSuccess) return e;
            (void)hipFree(b.ptr);
            b.ptr = nullptr;
            b.size = 0;
        }
        size_t want = bytes < (size_t)(32u << 20) ? (size_t)(32u << 20) : bytes;
        if ((e = hipMalloc(&b.ptr, want)) != hipSuccess) return e;
        b.size = want;
    }
    *out = static_cast<float*>(b.ptr);
    return hipSuccess;
}

}  // namespace pda

extern "C" {

const char* pda_last_error(void) { return g_err; }

int pda_version(void) { return 100; }

int pda_attn_fwd(const void* q, const void* k, const void* v, float* out, float* lse,
                 int B, int H, int64_t Sq, int64_t Skv, int d, float scale,
                 int64_t kv_valid_len, int64_t q_offset, void* stream) {
    int rc = check_attn_args(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len);
    if (rc != PDA_OK) return rc;
    if (q_offset < 0) return fail(PDA_ERR_INVALID_ARG, "q_offset=%lld is negative", (long long)q_offset);
    if (B == 0 || H == 0 || Sq == 0) return PDA_OK;
    hipError_t e = launch_heads(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, 0, H,
                                static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "attention launch");
    return PDA_OK;
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
    if (compute_stream == drain_stream) return fail(PDA_ERR_INVALID_ARG, "compute and drain streams must differ");
    if (sink && !aligned16(sink)) return fail(PDA_ERR_UNSUPPORTED, "sink must be 16-byte aligned");
    if (sink && sink == out) return fail(PDA_ERR_INVALID_ARG, "sink must not alias out");
    const int n_groups = H > 0 ? (H + heads_per_group - 1) / heads_per_group : 0;
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

    for (int g = 0; g < n_groups; ++g) {
        const int h0 = g * heads_per_group;
        const int hg = (h0 + heads_per_group <= H) ? heads_per_group : H - h0;
        if (timed && (e = hipEventRecord(beg[g], cs)) != hipSuccess) break;
        if ((e = launch_heads(q, k, v, out, lse, B, H, Sq, Skv, d, scale, kv_valid_len, h0, hg, cs)) != hipSuccess) break;
        if ((e = hipEventRecord(done[g], cs)) != hipSuccess) break;
        if ((e = hipStreamWaitEvent(ds, done[g], 0)) != hipSuccess) break;
        if (sink) {
            // hand-off of this group's result: its slice of out goes to the same slice of sink
            for (int b = 0; b < B && e == hipSuccess; ++b) {
                const int64_t off = ((int64_t)b * H + h0) * Sq * d;
                e = pda::launch_copy_f32(out + off, sink + off, (int64_t)hg * Sq * d, ds);
            }
            if (e != hipSuccess) break;
        }
    }
    if (e == hipSuccess && timed) e = hipEventRecord(drain_end, ds);
    if (e != hipSuccess) {
        (void)hipStreamSynchronize(cs);
        (void)hipStreamSynchronize(ds);
        cleanup();
        return hip_fail(e, "head-chunk pipeline");
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

}  // extern "C"
