// Host side of the C ABI declared in include/tsq.h: validation, blob layout,
// launch geometry, and the order of kernel launches.  No arithmetic of the
// method happens here except the translation of tau into a 16-bit pattern.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "tsq.h"
#include "tsq_measure.h"
#include "tsq_ranges.h"
#include "tsq_internal.hpp"
#include "tsq_ranges.hpp"

using namespace tsq;

struct tsq_plan {
    tsq_config cfg;
    Params p;
    Geometry g;
    EntropyLayout e;
    tsq_layout layout;
    int pipeline;  // resolved: TSQ_PIPE_STAGED or TSQ_PIPE_FUSED
};

namespace {

constexpr int kStaticMaxDevicesForOrder = 64;

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// value of a non-negative 16-bit pattern (sign bit clear), exact in double
double pattern_value(uint32_t pat, int dtype) {
    if (dtype == TSQ_BF16) {
        uint32_t u = pat << 16;
        float f;
        std::memcpy(&f, &u, 4);
        return (double)f;
    }
    const uint32_t e = (pat >> 10) & 0x1Fu, f = pat & 0x3FFu;
    if (e == 31) return f ? NAN : INFINITY;
    if (e == 0) return std::ldexp((double)f, -24);
    return std::ldexp((double)(1024 + f), (int)e - 25);
}

// Smallest magnitude pattern whose value is >= tau.  The pattern of +Inf always qualifies, so
// Inf and NaN (patterns above it) are on the outlier side for every finite tau.
uint32_t threshold_pattern(float tau, int dtype) {
    uint32_t lo = 0, hi = dtype == TSQ_BF16 ? 0x7F80u : 0x7C00u;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) / 2;
        if (pattern_value(mid, dtype) >= (double)tau) hi = mid; else lo = mid + 1;
    }
    return lo;
}

uint32_t row_bytes_host(uint32_t H, uint32_t b) { return 4u * ((H * b + 31u) / 32u); }

std::once_flag g_prepare_once;
int g_prepare_rc = 0;

tsq_status hip_rc(int e) { return e == 0 ? TSQ_OK : TSQ_ERR_HIP; }

}  // namespace

extern "C" {

const char *tsq_status_string(tsq_status s) {
    switch (s) {
        case TSQ_OK: return "ok";
        case TSQ_ERR_INVALID_ARG: return "invalid argument";
        case TSQ_ERR_UNSUPPORTED: return "unsupported shape or option";
        case TSQ_ERR_CAPACITY: return "outlier side stream exceeds max_outliers";
        case TSQ_ERR_HIP: return "HIP call failed";
        case TSQ_ERR_FORMAT: return "blob does not match this plan";
        case TSQ_ERR_INTERNAL: return "device-side wait expired";
        case TSQ_ERR_NO_MEMORY: return "host allocation failed";
    }
    return "unknown status";
}

tsq_status tsq_plan_create(const tsq_config *cfg, tsq_plan **out) {
    if (!cfg || !out) return TSQ_ERR_INVALID_ARG;
    if (cfg->tokens == 0 || cfg->hidden == 0) return TSQ_ERR_INVALID_ARG;
    if (cfg->dtype != TSQ_F16 && cfg->dtype != TSQ_BF16) return TSQ_ERR_INVALID_ARG;
    if (!(cfg->tau > 0.0f) || std::isinf(cfg->tau)) return TSQ_ERR_INVALID_ARG;
    if ((cfg->bit_mask & 0x1FCu) == 0 || (cfg->bit_mask & ~0x1FCu) != 0) return TSQ_ERR_INVALID_ARG;
    if (!(cfg->budget >= 0.0f)) return TSQ_ERR_INVALID_ARG;  // rejects NaN too
    if (cfg->mode != TSQ_BUDGET_LSB && cfg->mode != TSQ_BUDGET_REL_RMS) return TSQ_ERR_INVALID_ARG;
    if (cfg->pipeline < TSQ_PIPE_AUTO || cfg->pipeline > TSQ_PIPE_FUSED) return TSQ_ERR_INVALID_ARG;
    if (cfg->return_rule != TSQ_RETURN_LAST_PASSING && cfg->return_rule != TSQ_RETURN_AS_PRINTED) return TSQ_ERR_INVALID_ARG;
    if (cfg->reserved != 0) return TSQ_ERR_INVALID_ARG;
    if ((uint64_t)cfg->tokens * cfg->hidden >= (1ull << 32)) return TSQ_ERR_INVALID_ARG;
    if (cfg->hidden % 8 != 0 || cfg->hidden > kMaxHidden) return TSQ_ERR_UNSUPPORTED;

    tsq_plan *pl = new (std::nothrow) tsq_plan();
    if (!pl) return TSQ_ERR_NO_MEMORY;
    pl->cfg = *cfg;
    const uint32_t T = cfg->tokens, H = cfg->hidden;

    Params &p = pl->p;
    std::memset(&p, 0, sizeof p);
    p.tokens = T;
    p.hidden = H;
    p.runs = (H + kRun - 1) / kRun;
    p.pieces = H / 8;
    p.dtype = (uint32_t)cfg->dtype;
    const uint32_t thr = threshold_pattern(cfg->tau, cfg->dtype);
    p.thr_pk = thr | (thr << 16);
    p.bit_mask = cfg->bit_mask;
    uint32_t bmax = 0;
    for (int b = 8; b >= 2; --b)
        if (cfg->bit_mask & (1u << b)) {
            if (!bmax) bmax = (uint32_t)b;
            p.widths_pk |= (uint64_t)b << (8 * p.n_widths);
            ++p.n_widths;
        }
    for (uint32_t i = 0; i < p.n_widths; ++i) {
        const uint32_t Qi = (1u << (width_at(p, i) - 1u)) - 1u;
        if (cfg->mode == TSQ_BUDGET_LSB) {
            p.test_rhs[i] = (double)cfg->budget * (double)H;
        } else {
            double R = (double)cfg->budget * (double)Qi;
            R *= R;
            R *= (double)H;
            p.test_rhs[i] = R;
        }
    }
    p.tau = cfg->tau;
    p.budget = cfg->budget;
    p.mode = cfg->mode;
    p.return_failing = cfg->return_rule == TSQ_RETURN_AS_PRINTED ? 1u : 0u;
    p.spin_limit = 1u << 20;

    tsq_layout &L = pl->layout;
    uint64_t off = align_up(sizeof(BlobHeader), 256);
    L.off_bits = off;      off = align_up(off + T, 256);
    L.off_scale = off;     off = align_up(off + 4ull * T, 256);
    L.off_pay_off = off;   off = align_up(off + 8ull * (T + 1ull), 256);
    L.off_row_ptr = off;   off = align_up(off + 8ull * (T + 1ull), 256);
    L.payload_capacity = (uint64_t)T * row_bytes_host(H, bmax);
    L.off_payload = off;   off = align_up(off + L.payload_capacity, 256);
    L.outlier_capacity = cfg->max_outliers ? cfg->max_outliers : (uint64_t)T * H;
    if (L.outlier_capacity > (uint64_t)T * H) L.outlier_capacity = (uint64_t)T * H;
    L.off_out_col = off;   off = align_up(off + 2ull * L.outlier_capacity, 256);
    L.off_out_val = off;   off = align_up(off + 2ull * L.outlier_capacity, 256);
    L.blob_bytes = off;

    // the control block and the counters come first: they lie at the same place whatever the shape, so a
    // kernel can tell a workspace of another shape before it touches anything that depends on the shape
    uint64_t w = 0;
    p.ws_ctrl = w;   w = align_up(w + 256, 256);
    p.ws_tickets = w; w = align_up(w + 4ull * kTicketClasses * kTicketStride, 256);
    p.ws_cnt = w;    w = align_up(w + 4ull * T, 256);
    p.ws_amax = w;   w = align_up(w + 4ull * T, 256);
    p.ws_sizes = w;  w = align_up(w + 4ull * T, 256);
    p.ws_prefix = w; w = align_up(w + 8ull * (T + 1ull), 256);
    L.workspace_bytes = w;

    p.off_bits = L.off_bits; p.off_scale = L.off_scale; p.off_pay_off = L.off_pay_off;
    p.off_row_ptr = L.off_row_ptr; p.off_payload = L.off_payload; p.off_out_col = L.off_out_col;
    p.off_out_val = L.off_out_val; p.payload_capacity = L.payload_capacity;
    p.outlier_capacity = L.outlier_capacity;

    EntropyLayout &E = pl->e;
    std::memset(&E, 0, sizeof E);
    E.slot_bytes = 256u + 2u * ((H + 1u) & ~1u);     // 64 states, and at most one 16-bit word per element
    uint64_t eo = sizeof(EntropyHeader);
    E.off_tables = eo;      eo = align_up(eo + 7ull * 256 * 2, 256);
    E.off_stream_off = eo;  eo = align_up(eo + 8ull * (T + 1ull), 256);
    E.stream_capacity = (uint64_t)T * E.slot_bytes;
    E.off_streams = eo;     eo = align_up(eo + E.stream_capacity, 256);
    E.eblob_bytes = eo;
    uint64_t ew = 0;
    E.pool_tokens = (T + kMaxPoolGroups - 1u) / kMaxPoolGroups;
    if (E.pool_tokens < 16u) E.pool_tokens = 16u;    // a token per wave of a counting workgroup
    E.pool_groups = (T + E.pool_tokens - 1u) / E.pool_tokens;
    E.ws_pooled = ew;  ew = align_up(ew + (uint64_t)kPoolCopies * 7ull * 256 * 4, 256);
    E.ws_block = ew;   ew = align_up(ew + 4ull * kBlockStride * ((T + kLenBlock - 1u) / kLenBlock), 256);
    E.ws_len = ew;     ew = align_up(ew + 4ull * T, 256);
    E.ws_slots = ew;   ew = align_up(ew + (uint64_t)T * E.slot_bytes, 256);
    E.ws_bytes = ew;

    pl->g.block = 64u * ((p.runs + 63u) / 64u);
    pl->g.lds_bytes = (p.runs * kRunLdsDw + kScratchDw) * 4u;
    pl->g.waves = compress_waves(p.runs);
    // row 16 + two images 8 dwords per run, reduce areas and ticket slots, two stashes per wave
    pl->g.lds_fused_bytes = (p.runs * 32u + kFusedScratchDw + 2u * pl->g.waves * kStashWave) * 4u;
    pl->pipeline = cfg->pipeline == TSQ_PIPE_STAGED ? TSQ_PIPE_STAGED : TSQ_PIPE_FUSED;
    *out = pl;
    return TSQ_OK;
}

void tsq_plan_destroy(tsq_plan *plan) { delete plan; }

tsq_status tsq_plan_layout(const tsq_plan *plan, tsq_layout *out) {
    if (!plan || !out) return TSQ_ERR_INVALID_ARG;
    *out = plan->layout;
    return TSQ_OK;
}

size_t tsq_plan_blob_bytes(const tsq_plan *plan) { return plan ? (size_t)plan->layout.blob_bytes : 0; }
size_t tsq_plan_workspace_bytes(const tsq_plan *plan) { return plan ? (size_t)plan->layout.workspace_bytes : 0; }

static tsq_status ensure_prepared() {
    std::call_once(g_prepare_once, [] {
        g_prepare_rc = prepare_kernels();
        if (g_prepare_rc == 0) g_prepare_rc = prepare_fused_kernels();
    });
    return hip_rc(g_prepare_rc);
}

// Computing workgroups of the fused kernel: as many as the device holds at once next to the scanner
// workgroup (more would only queue up behind them), and no more than there are tokens.
static tsq_status fused_grid(const tsq_plan *plan, uint32_t *grid) {
    uint32_t resident = 0;
    const int rc = fused_resident_workgroups(plan->p, plan->g, &resident);
    if (rc != 0) return TSQ_ERR_HIP;
    uint32_t g = resident > 1 ? resident - 1 : 0;       // 0: scanner and computing workgroup do not both fit
    if (g > kFusedGridCap) g = kFusedGridCap;
    if (g > plan->p.tokens) g = plan->p.tokens;
    *grid = g;
    return TSQ_OK;
}

tsq_status tsq_workspace_reset(const tsq_plan *plan, void *d_ws, void *stream) {
    if (!plan || !d_ws) return TSQ_ERR_INVALID_ARG;
    return hip_rc(launch_ws_reset(plan->p, d_ws, stream));
}

// Single-pass compress kernels of different streams must not share the device.  Such a kernel's workgroups
// wait for one another (for a token's place, which needs every token before it); one kernel alone always gets
// all the workgroups it needs to run, but two of them, each holding compute-unit slots that the other one's
// not yet started workgroups need, can keep each other waiting until the bounded waits expire.  So the
// library orders them: a call on another stream than the previous call's (on the same device) first makes its
// stream wait for what the previous call's stream holds at that moment (an event recorded at its end).  Calls
// that stay on one stream pay nothing for this.  Under stream capture nothing is recorded: the calls of one
// captured graph are ordered by the graph.
struct FusedOrder {
    hipEvent_t tail = nullptr;          // recorded at the end of last_stream when the stream changes
    hipStream_t last_stream = nullptr;
    bool any = false;
};
static std::mutex g_order_mutex;
static FusedOrder g_order[kStaticMaxDevicesForOrder];

static bool is_capturing(hipStream_t s) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
    return st != hipStreamCaptureStatusNone;
}

static int launch_fused_ordered(const Params &p, const Geometry &g, uint32_t grid, const void *d_in, void *d_blob,
                                void *d_ws, void *stream) {
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    int dev = -1;
    if (is_capturing(s) || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevicesForOrder)
        return launch_fused(p, g, grid, d_in, d_blob, d_ws, stream);
    std::lock_guard<std::mutex> lock(g_order_mutex);
    FusedOrder &o = g_order[dev];
    if (o.any && o.last_stream != s && !is_capturing(o.last_stream)) {
        if (!o.tail && hipEventCreateWithFlags(&o.tail, hipEventDisableTiming) != hipSuccess) return (int)hipGetLastError();
        // (a stream that its owner has destroyed in the meantime cannot hold unfinished work: errors are dropped)
        if (hipEventRecord(o.tail, o.last_stream) == hipSuccess) {
            const hipError_t e = hipStreamWaitEvent(s, o.tail, 0);
            if (e != hipSuccess) return (int)e;
        } else {
            (void)hipGetLastError();
        }
    }
    const int rc = launch_fused(p, g, grid, d_in, d_blob, d_ws, stream);
    if (rc == 0) { o.last_stream = s; o.any = true; }
    return rc;
}

// One compress call.  rows_per_tensor == 0: d_in is the tensor; otherwise d_in is a device table of
// tensor pointers (the kernels pick the row's tensor from it).
static tsq_status compress_call(const tsq_plan *plan, const void *d_in, uint32_t rows_per_tensor, void *d_blob,
                                void *d_ws, void *stream, bool force_staged = false) {
    tsq_status st = ensure_prepared();
    if (st != TSQ_OK) return st;
    Params p = plan->p;
    p.rows_per_tensor = rows_per_tensor;
    if (plan->pipeline == TSQ_PIPE_FUSED && !force_staged) {
        uint32_t grid = 0;
        st = fused_grid(plan, &grid);
        // TSQ_PIPE_AUTO: a device that cannot tell how many workgroups it holds, or holds fewer than the
        // scanner and one computing workgroup, gets the staged pipeline, which needs nothing resident
        const bool fits = st == TSQ_OK && grid >= 1;
        if (!fits && plan->cfg.pipeline != TSQ_PIPE_AUTO) return st != TSQ_OK ? st : TSQ_ERR_UNSUPPORTED;
        if (fits) {
            p.fused_classes = grid < kTicketClasses ? grid : kTicketClasses;
            return hip_rc(launch_fused_ordered(p, plan->g, grid, d_in, d_blob, d_ws, stream));
        }
    }
    int e = launch_row_stats(p, plan->g, d_in, d_blob, d_ws, stream);
    if (e == 0) e = launch_scan(p, d_blob, d_ws, stream);
    if (e == 0) e = launch_pack(p, plan->g, d_in, d_blob, d_ws, stream);
    return hip_rc(e);
}

tsq_status tsq_compress(const tsq_plan *plan, const void *d_in, void *d_blob, void *d_ws, void *stream) {
    if (!plan || !d_in || !d_blob || !d_ws) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_in & 15u) || ((uintptr_t)d_blob & 255u) || ((uintptr_t)d_ws & 255u)) return TSQ_ERR_INVALID_ARG;
    return compress_call(plan, d_in, 0, d_blob, d_ws, stream);
}

// ---- tsq_compress for callers that cannot allocate: the workspace is a static device array.
// `scratch` is a host-side stand-in for the array, not a device address: every use below goes
// through the pointer that hipGetSymbolAddress returned for the device at hand.
constexpr size_t kStaticWorkspaceBytes = 4u << 20;
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) uint8_t scratch[kStaticWorkspaceBytes];
static std::mutex g_static_mutex;
static void *g_static_ws[kStaticMaxDevices];        // per device: where that device holds its copy of `scratch`

// The current device's copy of the array (looked up once per device, with that device current).
static tsq_status static_workspace(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return TSQ_ERR_HIP;
    if (dev < 0 || dev >= kStaticMaxDevices) return TSQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ws[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TSQ_ERR_HIP;
        g_static_ws[dev] = ptr;
    }
    *out = g_static_ws[dev];
    return TSQ_OK;
}

size_t tsq_static_workspace_bytes(void) { return kStaticWorkspaceBytes; }

tsq_status tsq_compress_static(const tsq_plan *plan, const void *d_in, void *d_blob, void *stream) {
    if (!plan || !d_in || !d_blob) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_in & 15u) || ((uintptr_t)d_blob & 255u)) return TSQ_ERR_INVALID_ARG;
    if (plan->layout.workspace_bytes > kStaticWorkspaceBytes) return TSQ_ERR_UNSUPPORTED;
    void *ws = nullptr;
    tsq_status st = static_workspace(&ws);
    if (st != TSQ_OK) return st;
    // the array keeps what the last call (of any plan) left in it: a small fill kernel puts the part this
    // plan uses back into its initial state (a kernel, not a memset, so that the call can be captured)
    if (launch_ws_reset(plan->p, ws, stream) != 0) return TSQ_ERR_HIP;
    return compress_call(plan, d_in, 0, d_blob, ws, stream);
}

tsq_status tsq_compress_batch(const tsq_plan *plan, const void *const *d_in_ptrs, uint32_t rows_per_tensor,
                              void *d_blob, void *d_ws, void *stream) {
    if (!plan || !d_in_ptrs || !d_blob || !d_ws) return TSQ_ERR_INVALID_ARG;
    if (rows_per_tensor == 0 || plan->p.tokens % rows_per_tensor != 0) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_in_ptrs & 7u) || ((uintptr_t)d_blob & 255u) || ((uintptr_t)d_ws & 255u)) return TSQ_ERR_INVALID_ARG;
    return compress_call(plan, d_in_ptrs, rows_per_tensor, d_blob, d_ws, stream);
}

tsq_status tsq_compress_timed(const tsq_plan *plan, const void *d_in, void *d_blob, void *d_ws, void *stream,
                              float *ms_out) {
    if (!plan || !d_in || !d_blob || !d_ws || !ms_out) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_in & 15u) || ((uintptr_t)d_blob & 255u) || ((uintptr_t)d_ws & 255u)) return TSQ_ERR_INVALID_ARG;
    tsq_status st = ensure_prepared();
    if (st != TSQ_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t ev[4];
    for (int i = 0; i < 4; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            while (i > 0) (void)hipEventDestroy(ev[--i]);
            return TSQ_ERR_HIP;
        }
    int rc = 0, n = 0;
    (void)hipEventRecord(ev[0], s);
    if (plan->pipeline == TSQ_PIPE_FUSED) {
        uint32_t grid = 0;
        st = fused_grid(plan, &grid);
        Params p = plan->p;
        p.fused_classes = grid < kTicketClasses ? grid : kTicketClasses;
        if (st == TSQ_OK && grid >= 1) rc = launch_fused(p, plan->g, grid, d_in, d_blob, d_ws, stream); else rc = 1;
        (void)hipEventRecord(ev[1], s);
        n = 1;
    } else {
        rc = launch_row_stats(plan->p, plan->g, d_in, d_blob, d_ws, stream);
        (void)hipEventRecord(ev[1], s);
        if (rc == 0) rc = launch_scan(plan->p, d_blob, d_ws, stream);
        (void)hipEventRecord(ev[2], s);
        if (rc == 0) rc = launch_pack(plan->p, plan->g, d_in, d_blob, d_ws, stream);
        (void)hipEventRecord(ev[3], s);
        n = 3;
    }
    if (hipEventSynchronize(ev[n]) != hipSuccess) rc = rc ? rc : 1;
    for (int i = 0; i < 4; ++i) ms_out[i] = 0.0f;
    for (int i = 0; i < n && rc == 0; ++i)
        if (hipEventElapsedTime(&ms_out[i], ev[i], ev[i + 1]) != hipSuccess) rc = 1;
    for (auto &e : ev) (void)hipEventDestroy(e);
    return hip_rc(rc);
}

tsq_status tsq_decompress(const tsq_plan *plan, const void *d_blob, void *d_out, void *stream) {
    if (!plan || !d_blob || !d_out) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_out & 15u) || ((uintptr_t)d_blob & 255u)) return TSQ_ERR_INVALID_ARG;
    tsq_status st = ensure_prepared();
    if (st != TSQ_OK) return st;
    return hip_rc(launch_unpack(plan->p, plan->g, d_blob, d_out, stream));
}

tsq_status tsq_decompress_batch(const tsq_plan *plan, const void *d_blob, void *const *d_out_ptrs,
                                uint32_t rows_per_tensor, void *stream) {
    if (!plan || !d_blob || !d_out_ptrs) return TSQ_ERR_INVALID_ARG;
    if (rows_per_tensor == 0 || plan->p.tokens % rows_per_tensor != 0) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_out_ptrs & 7u) || ((uintptr_t)d_blob & 255u)) return TSQ_ERR_INVALID_ARG;
    tsq_status st = ensure_prepared();
    if (st != TSQ_OK) return st;
    Params p = plan->p;
    p.rows_per_tensor = rows_per_tensor;
    return hip_rc(launch_unpack(p, plan->g, d_blob, const_cast<void **>(d_out_ptrs), stream));
}

tsq_status tsq_code_histogram(const tsq_plan *plan, const void *d_blob, void *d_hist, void *stream) {
    if (!plan || !d_blob || !d_hist) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_hist & 3u) || ((uintptr_t)d_blob & 255u)) return TSQ_ERR_INVALID_ARG;
    return hip_rc(launch_code_hist(plan->p, plan->g, d_blob, d_hist, stream));
}

size_t tsq_entropy_blob_bytes(const tsq_plan *plan) { return plan ? (size_t)plan->e.eblob_bytes : 0; }
size_t tsq_entropy_workspace_bytes(const tsq_plan *plan) { return plan ? (size_t)plan->e.ws_bytes : 0; }

tsq_status tsq_entropy_encode(const tsq_plan *plan, const void *d_blob, void *d_eblob, void *d_ews, void *stream) {
    if (!plan || !d_blob || !d_eblob || !d_ews) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_blob & 255u) || ((uintptr_t)d_eblob & 255u) || ((uintptr_t)d_ews & 255u)) return TSQ_ERR_INVALID_ARG;
    tsq_status st = ensure_prepared();
    if (st != TSQ_OK) return st;
    return hip_rc(launch_rans_encode(plan->p, plan->g, plan->e, d_blob, d_eblob, d_ews, stream));
}

tsq_status tsq_entropy_decode(const tsq_plan *plan, const void *d_eblob, void *d_blob, void *stream) {
    if (!plan || !d_blob || !d_eblob) return TSQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_blob & 255u) || ((uintptr_t)d_eblob & 255u)) return TSQ_ERR_INVALID_ARG;
    tsq_status st = ensure_prepared();
    if (st != TSQ_OK) return st;
    return hip_rc(launch_rans_decode(plan->p, plan->e, d_eblob, d_blob, stream));
}

tsq_status tsq_entropy_info(const tsq_plan *plan, const void *d_eblob, tsq_entropy_layout *host_out, void *stream) {
    if (!plan || !d_eblob || !host_out) return TSQ_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    EntropyHeader h;
    if (hipMemcpyAsync(&h, d_eblob, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return TSQ_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return TSQ_ERR_HIP;
    std::memset(host_out, 0, sizeof *host_out);
    const EntropyLayout &E = plan->e;
    host_out->off_tables = E.off_tables; host_out->off_stream_off = E.off_stream_off;
    host_out->off_streams = E.off_streams; host_out->stream_capacity = E.stream_capacity;
    if (h.magic != kEntropyMagic || h.version != kVersion || h.tokens != plan->p.tokens || h.hidden != plan->p.hidden ||
        h.off_streams != E.off_streams || h.stream_bytes > E.stream_capacity)
        return TSQ_ERR_FORMAT;
    host_out->stream_bytes = h.stream_bytes;
    host_out->coded_bytes = 256ull + 7ull * 256 * 2 + 8ull * (plan->p.tokens + 1ull) + h.stream_bytes;
    return TSQ_OK;
}

tsq_status tsq_blob_info(const tsq_plan *plan, const void *d_blob, tsq_info *host_out, void *stream) {
    if (!plan || !d_blob || !host_out) return TSQ_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    BlobHeader h;
    const Params &p = plan->p;
    struct Bytes {                                   // host buffer that cannot throw
        uint8_t *at;
        explicit Bytes(size_t n) : at(static_cast<uint8_t *>(std::malloc(n ? n : 1))) {}
        ~Bytes() { std::free(at); }
    } bits(p.tokens);
    if (!bits.at) return TSQ_ERR_NO_MEMORY;
    if (hipMemcpyAsync(&h, d_blob, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return TSQ_ERR_HIP;
    if (hipMemcpyAsync(bits.at, static_cast<const uint8_t *>(d_blob) + plan->layout.off_bits, p.tokens,
                       hipMemcpyDeviceToHost, s) != hipSuccess) {
        (void)hipStreamSynchronize(s);               // the first copy may still be writing into h
        return TSQ_ERR_HIP;
    }
    if (hipStreamSynchronize(s) != hipSuccess) return TSQ_ERR_HIP;
    std::memset(host_out, 0, sizeof *host_out);
    if (h.magic != kMagic || h.version != kVersion || h.tokens != p.tokens || h.hidden != p.hidden ||
        h.dtype != p.dtype || h.bit_mask != p.bit_mask || h.off_payload != p.off_payload ||
        h.off_out_col != p.off_out_col || h.off_out_val != p.off_out_val)
        return TSQ_ERR_FORMAT;
    host_out->status = h.status;
    host_out->nnz = h.nnz;
    host_out->payload_bytes = h.payload_bytes;
    host_out->compressed_bytes = 128ull + 5ull * p.tokens + 16ull * (p.tokens + 1ull) + h.payload_bytes + 4ull * h.nnz;
    for (uint32_t t = 0; t < p.tokens; ++t)
        if (bits.at[t] <= 8) host_out->width_hist[bits.at[t]]++;
    if (h.status == TSQ_ERR_CAPACITY) return TSQ_ERR_CAPACITY;
    if (h.status == TSQ_ERR_FORMAT) return TSQ_ERR_FORMAT;      // the workspace was another shape's, or never reset
    if (h.status != 0) return TSQ_ERR_INTERNAL;
    return TSQ_OK;
}

tsq_status tsq_prefix_bytes(const tsq_plan *plan, const void *d_blob, const uint32_t *k, uint32_t n, uint64_t *bytes_out,
                            void *stream) {
    if (!plan || !d_blob || n == 0 || !bytes_out) return TSQ_ERR_INVALID_ARG;
    const Params &p = plan->p;
    if (!k && (uint64_t)n > p.tokens + 1ull) return TSQ_ERR_INVALID_ARG;
    for (uint32_t i = 0; k && i < n; ++i)
        if (k[i] > p.tokens) return TSQ_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const uint8_t *blob = static_cast<const uint8_t *>(d_blob);
    BlobHeader h;
    if (hipMemcpyAsync(&h, blob, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return TSQ_ERR_HIP;
    // bytes_out doubles as the landing place of pay_off[k]; row_ptr[k] lands in a buffer of its own
    uint64_t *rp = static_cast<uint64_t *>(std::malloc(sizeof(uint64_t) * n));
    if (!rp) { (void)hipStreamSynchronize(s); return TSQ_ERR_NO_MEMORY; }
    int bad = 0;
    if (!k) {       // k = 0 .. n-1: the tables' first n entries in one copy each
        bad |= hipMemcpyAsync(bytes_out, blob + p.off_pay_off, 8ull * n, hipMemcpyDeviceToHost, s) != hipSuccess;
        bad |= hipMemcpyAsync(rp, blob + p.off_row_ptr, 8ull * n, hipMemcpyDeviceToHost, s) != hipSuccess;
    }
    for (uint32_t i = 0; k && i < n && !bad; ++i) {
        bad |= hipMemcpyAsync(&bytes_out[i], blob + p.off_pay_off + 8ull * k[i], 8, hipMemcpyDeviceToHost, s) != hipSuccess;
        bad |= hipMemcpyAsync(&rp[i], blob + p.off_row_ptr + 8ull * k[i], 8, hipMemcpyDeviceToHost, s) != hipSuccess;
    }
    if (hipStreamSynchronize(s) != hipSuccess) bad = 1;
    tsq_status st = bad ? TSQ_ERR_HIP : TSQ_OK;
    if (st == TSQ_OK && (h.magic != kMagic || h.version != kVersion || h.tokens != p.tokens || h.hidden != p.hidden ||
                         h.off_pay_off != p.off_pay_off || h.off_row_ptr != p.off_row_ptr))
        st = TSQ_ERR_FORMAT;
    if (st == TSQ_OK && h.status != 0) st = h.status == TSQ_ERR_CAPACITY ? TSQ_ERR_CAPACITY : TSQ_ERR_INTERNAL;
    // header + per-token metadata of k tokens (5 bytes and two offsets each, one closing pair) + codes + CSR entries
    for (uint32_t i = 0; i < n && st == TSQ_OK; ++i) {
        const uint64_t ki = k ? k[i] : i;
        bytes_out[i] = 128ull + 5ull * ki + 16ull * (ki + 1ull) + bytes_out[i] + 4ull * rp[i];
    }
    std::free(rp);
    return st;
}

tsq_status tsq_entropy_prefix_bytes(const tsq_plan *plan, const void *d_blob, const void *d_eblob, const uint32_t *k,
                                    uint32_t n, uint64_t *bytes_out, void *stream) {
    if (!plan || !d_blob || !d_eblob || n == 0 || !bytes_out) return TSQ_ERR_INVALID_ARG;
    const Params &p = plan->p;
    const EntropyLayout &E = plan->e;
    if (!k && (uint64_t)n > p.tokens + 1ull) return TSQ_ERR_INVALID_ARG;
    for (uint32_t i = 0; k && i < n; ++i)
        if (k[i] > p.tokens) return TSQ_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const uint8_t *blob = static_cast<const uint8_t *>(d_blob), *eblob = static_cast<const uint8_t *>(d_eblob);
    BlobHeader h;
    EntropyHeader eh;
    if (hipMemcpyAsync(&h, blob, sizeof h, hipMemcpyDeviceToHost, s) != hipSuccess) return TSQ_ERR_HIP;
    if (hipMemcpyAsync(&eh, eblob, sizeof eh, hipMemcpyDeviceToHost, s) != hipSuccess) {
        (void)hipStreamSynchronize(s);
        return TSQ_ERR_HIP;
    }
    // bytes_out doubles as the landing place of the stream offsets; row_ptr[k] lands in a buffer of its own
    uint64_t *rp = static_cast<uint64_t *>(std::malloc(sizeof(uint64_t) * n));
    if (!rp) { (void)hipStreamSynchronize(s); return TSQ_ERR_NO_MEMORY; }
    int bad = 0;
    if (!k) {
        bad |= hipMemcpyAsync(bytes_out, eblob + E.off_stream_off, 8ull * n, hipMemcpyDeviceToHost, s) != hipSuccess;
        bad |= hipMemcpyAsync(rp, blob + p.off_row_ptr, 8ull * n, hipMemcpyDeviceToHost, s) != hipSuccess;
    }
    for (uint32_t i = 0; k && i < n && !bad; ++i) {
        bad |= hipMemcpyAsync(&bytes_out[i], eblob + E.off_stream_off + 8ull * k[i], 8, hipMemcpyDeviceToHost, s) != hipSuccess;
        bad |= hipMemcpyAsync(&rp[i], blob + p.off_row_ptr + 8ull * k[i], 8, hipMemcpyDeviceToHost, s) != hipSuccess;
    }
    if (hipStreamSynchronize(s) != hipSuccess) bad = 1;
    tsq_status st = bad ? TSQ_ERR_HIP : TSQ_OK;
    if (st == TSQ_OK && (h.magic != kMagic || h.version != kVersion || h.tokens != p.tokens || h.hidden != p.hidden ||
                         h.off_row_ptr != p.off_row_ptr))
        st = TSQ_ERR_FORMAT;
    if (st == TSQ_OK && h.status != 0) st = h.status == TSQ_ERR_CAPACITY ? TSQ_ERR_CAPACITY : TSQ_ERR_INTERNAL;
    if (st == TSQ_OK && (eh.magic != kEntropyMagic || eh.version != kVersion || eh.tokens != p.tokens || eh.hidden != p.hidden ||
                         eh.off_streams != E.off_streams || eh.stream_bytes > E.stream_capacity))
        st = TSQ_ERR_FORMAT;
    // the blob's header and per-token metadata of k tokens and its CSR entries, as in tsq_prefix_bytes; in place of the
    // codes: the coded blob's header, its tables, k + 1 stream offsets and the streams before offset[k]
    for (uint32_t i = 0; i < n && st == TSQ_OK; ++i) {
        const uint64_t ki = k ? k[i] : i;
        if (bytes_out[i] > eh.stream_bytes) { st = TSQ_ERR_FORMAT; break; }
        bytes_out[i] = 128ull + 5ull * ki + 16ull * (ki + 1ull) + 4ull * rp[i] +
                       sizeof(EntropyHeader) + 7ull * 256 * 2 + 8ull * (ki + 1ull) + bytes_out[i];
    }
    std::free(rp);
    return st;
}

tsq_status tsq_compress_blocking(const tsq_plan *plan, const void *d_in, void *d_blob, void *d_ws, void *stream,
                                 tsq_info *info_out) {
    if (!info_out) return TSQ_ERR_INVALID_ARG;
    tsq_status st = tsq_compress(plan, d_in, d_blob, d_ws, stream);
    if (st != TSQ_OK) return st;
    st = tsq_blob_info(plan, d_blob, info_out, stream);
    const bool workspace_trouble = st == TSQ_ERR_INTERNAL || (st == TSQ_ERR_FORMAT && info_out->status == TSQ_ERR_FORMAT);
    if (!workspace_trouble || plan->cfg.pipeline != TSQ_PIPE_AUTO || plan->pipeline != TSQ_PIPE_FUSED) return st;
    // the single pass gave up (a wait expired, or the workspace was not in its initial state): the same call
    // once more on a fresh workspace with the staged kernels, which wait for nothing
    st = tsq_workspace_reset(plan, d_ws, stream);
    if (st == TSQ_OK) st = compress_call(plan, d_in, 0, d_blob, d_ws, stream, true);
    if (st != TSQ_OK) return st;
    return tsq_blob_info(plan, d_blob, info_out, stream);
}

// ---- the kernels' range predicates, evaluated on the host (include/tsq_ranges.h)
int tsq_check_payload_span(uint32_t hidden, uint64_t capacity, uint32_t width, uint64_t offset) {
    return payload_span_ok(hidden, capacity, width, offset) ? 1 : 0;
}
int tsq_check_csr_slice(uint64_t rp0, uint64_t rp1, uint64_t capacity) { return csr_slice_ok(rp0, rp1, capacity) ? 1 : 0; }
int tsq_check_csr_slice_holds(uint64_t rp0, uint64_t rp1, uint64_t capacity, uint32_t count) {
    return csr_slice_holds(rp0, rp1, capacity, count) ? 1 : 0;
}
int tsq_check_column(uint32_t column, uint32_t hidden) { return column_ok(column, hidden) ? 1 : 0; }
int tsq_check_stream_span(uint64_t begin, uint64_t end, uint64_t capacity, uint32_t coders, uint32_t slot_bytes) {
    return stream_span_ok(begin, end, capacity, coders, slot_bytes) ? 1 : 0;
}
void tsq_check_quotients(const uint32_t *x, const uint32_t *f, uint32_t *q, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) q[i] = quotient_or_one_less(x[i], reciprocal_just_below(f[i]));
}
int tsq_check_stream_move(uint32_t bytes, uint32_t coders, uint32_t slot_bytes, uint64_t at, uint64_t capacity) {
    return stream_move_ok(bytes, coders, slot_bytes, at, capacity) ? 1 : 0;
}
uint32_t tsq_check_frequency_slot(uint32_t state) { return frequency_slot(state); }
int tsq_check_workspace_shape(uint32_t ws_tokens, uint32_t ws_hidden, uint32_t tokens, uint32_t hidden) {
    return workspace_shape_ok(ws_tokens, ws_hidden, tokens, hidden) ? 1 : 0;
}

// ---- copy ceilings (include/tsq_measure.h)
tsq_status tsq_measure_copy(void *d_dst, const void *d_src, size_t bytes, void *stream) {
    if (!d_dst || !d_src || bytes == 0 || (bytes & 15u) || ((uintptr_t)d_dst & 15u) || ((uintptr_t)d_src & 15u))
        return TSQ_ERR_INVALID_ARG;
    return hip_rc(launch_plain_copy(d_dst, d_src, bytes, stream));
}
tsq_status tsq_measure_read(const void *d_src, size_t bytes, void *d_sink, void *stream) {
    if (!d_sink || !d_src || bytes == 0 || (bytes & 15u) || ((uintptr_t)d_src & 15u) || ((uintptr_t)d_sink & 3u))
        return TSQ_ERR_INVALID_ARG;
    return hip_rc(launch_plain_read(d_src, bytes, d_sink, stream));
}

}  // extern "C"
