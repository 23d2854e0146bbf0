// Row kernels, scan kernel and their launchers (gfx950).
//
//   k_row_stats : Eq. (ts) + Algorithm 1 per token -> width, scale, outlier count
//   k_scan      : exclusive scan of outlier counts and payload sizes -> CSR row
//                 pointers and payload offsets, blob header
//   k_pack      : Eq. (Proposed) at the chosen width, bit packing, CSR emission
//   k_unpack    : Eq. (dequnt): unpack, dequantize, outliers back in place
#include <hip/hip_runtime.h>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

// LDS map of the row kernels (dynamic):  [ row: runs*kRunLdsDw dwords | scratch: kScratchDw dwords ]
//   scratch: reduce area 0 [0,32) | reduce area 1 [32,64) | scan area [64,80) | broadcast area [80,88);
//   the scan workgroup of the fused kernel uses [0,96) as two areas of 3 dwords per wave
constexpr uint32_t kScrScan = 4 * kMaxWaves, kScrBcast = 5 * kMaxWaves;

__device__ __forceinline__ uint32_t row_bytes(uint32_t H, uint32_t b) { return 4u * ((H * b + 31u) >> 5); }

// ---------------------------------------------------------------- Algorithm 1 for the token of this block

struct Choice {
    uint32_t width;  // b_t
    float amax;      // inlier absmax
    uint32_t cnt;    // outliers in the token
};

// On return m holds the magnitude bytes of the run at the chosen width.
template <int DT>
__device__ __forceinline__ Choice choose_width(const Params &p, const uint32_t (&apk)[16], uint32_t omask,
                                               uint32_t amax_pk, uint32_t *scratch, uint32_t (&m)[8]) {
    float af[32];
    widen_run<DT>(apk, af);
    uint32_t *red0 = scratch, *red1 = scratch + 2 * kMaxWaves;
    uint32_t mx = (amax_pk & 0xFFFFu) > (amax_pk >> 16) ? (amax_pk & 0xFFFFu) : (amax_pk >> 16);
    uint32_t cnt = (uint32_t)__builtin_popcount(omask);
    block_max_sum(mx, cnt, red0);
    const float amax = widen16<DT>(mx);

    // lane k of every wave holds r = Q_k / amax of the k-th allowed width (one division per wave)
    const uint32_t lane = threadIdx.x & 63;
    float rq = 0.0f;
    if (lane < p.n_widths && amax >= kAmaxFloor) rq = level_count(width_at(p, lane)) / amax;

    const uint32_t b0 = width_at(p, 0);
    const uint32_t Q0 = (1u << (b0 - 1)) - 1u;
    quantize_run(af, __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(rq), 0)), m);
    uint32_t sel = b0;

    if (p.n_widths > 1) {
        uint32_t m0[8];
#pragma unroll
        for (int g = 0; g < 8; ++g) m0[g] = m[g];
        uint32_t ss0 = sum_squares_run(m0);
        for (uint32_t i = 1; i < p.n_widths; ++i) {
            const uint32_t bi = width_at(p, i);
            uint32_t mi[8];
            quantize_run(af, __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(rq), (int)i)), mi);
            uint32_t sad = sad_run(m0, mi, b0 - bi);
            if (i == 1) block_sum2(sad, ss0, red1); else block_sum1(sad, (i & 1) ? red1 : red0);
            if (violates(p.mode, p.budget, p.hidden, Q0, (1u << (bi - 1)) - 1u, sad, ss0)) break;
            sel = bi;
#pragma unroll
            for (int g = 0; g < 8; ++g) m[g] = mi[g];
        }
    }
    Choice c;
    c.width = sel;
    c.amax = amax;
    c.cnt = cnt;
    return c;
}

__device__ __forceinline__ float scale_of(float amax, uint32_t width) {
    return amax >= kAmaxFloor ? amax / level_count(width) : 0.0f;
}

// ---------------------------------------------------------------- payload + CSR output of one token

template <int B>
__device__ __forceinline__ void store_codes(const uint32_t (&m)[8], const uint32_t *lrun, uint32_t *dst_row,
                                            uint32_t run, uint32_t valid_pieces) {
    uint32_t out[B];
    pack_run<B>(m, lrun, out);
    uint32_t *dst = dst_row + run * B;
    if (valid_pieces >= 4) {
#pragma unroll
        for (int k = 0; k < B; ++k) dst[k] = out[k];
    } else {
        const uint32_t nd = (valid_pieces * B + 3u) >> 2;  // ceil(8*valid*B / 32)
#pragma unroll
        for (int k = 0; k < B; ++k)
            if ((uint32_t)k < nd) dst[k] = out[k];
    }
}

__device__ __forceinline__ void store_codes_any(uint32_t width, const uint32_t (&m)[8], const uint32_t *lrun,
                                                uint32_t *dst_row, uint32_t run, uint32_t valid_pieces) {
    switch (width) {
        case 2: store_codes<2>(m, lrun, dst_row, run, valid_pieces); break;
        case 3: store_codes<3>(m, lrun, dst_row, run, valid_pieces); break;
        case 4: store_codes<4>(m, lrun, dst_row, run, valid_pieces); break;
        case 5: store_codes<5>(m, lrun, dst_row, run, valid_pieces); break;
        case 6: store_codes<6>(m, lrun, dst_row, run, valid_pieces); break;
        case 7: store_codes<7>(m, lrun, dst_row, run, valid_pieces); break;
        default: store_codes<8>(m, lrun, dst_row, run, valid_pieces); break;
    }
}

// T_above of the token in CSR: ascending columns, raw values.  Lane order is column order,
// so a prefix sum over the lanes' outlier counts places every lane's outliers.
// Must be called by all threads of the block (contains a barrier).
__device__ __forceinline__ void emit_outliers(uint32_t omask, const uint32_t *lrow, uint32_t run, uint16_t *col,
                                              uint16_t *val, uint64_t row_start, uint32_t *scan_scr) {
    const uint32_t n = (uint32_t)__builtin_popcount(omask);
    uint64_t pos = row_start + block_excl_scan(n, scan_scr);
    uint32_t ev = omask & 0xFFFFu, od = omask >> 16;
    const uint16_t *raw = reinterpret_cast<const uint16_t *>(lrow + run * kRunLdsDw);
    while (ev | od) {
        const uint32_t je = ev ? 2u * (uint32_t)__builtin_ctz(ev) : 64u;
        const uint32_t jo = od ? 2u * (uint32_t)__builtin_ctz(od) + 1u : 64u;
        uint32_t j;
        if (je < jo) { j = je; ev &= ev - 1u; } else { j = jo; od &= od - 1u; }
        col[pos] = (uint16_t)(run * kRun + j);
        val[pos] = raw[j];
        ++pos;
    }
}

// ---------------------------------------------------------------- k_row_stats

template <int DT>
__global__ void __launch_bounds__(1024)
k_row_stats(const Params p, const uint16_t *__restrict__ in, uint8_t *__restrict__ blob, uint8_t *__restrict__ ws) {
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t *lrow = lds;
    uint32_t *scratch = lds + p.runs * kRunLdsDw;
    const uint32_t t = blockIdx.x;
    const uint32_t run = threadIdx.x;

    stage_row(reinterpret_cast<const uint4 *>(in + (size_t)t * p.hidden), p.pieces, p.runs, lrow);
    clear_reduce_areas(scratch);
    __syncthreads();

    uint32_t apk[16], omask = 0, amax_pk = 0;
    if (run < p.runs) {
        split_run<true>(lrow + run * kRunLdsDw, p.thr_pk, apk, omask, amax_pk);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) apk[i] = 0;
    }
    uint32_t m[8];
    const Choice c = choose_width<DT>(p, apk, omask, amax_pk, scratch, m);
    if (threadIdx.x == 0) {
        blob[p.off_bits + t] = (uint8_t)c.width;
        reinterpret_cast<float *>(blob + p.off_scale)[t] = scale_of(c.amax, c.width);
        reinterpret_cast<uint32_t *>(ws + p.ws_cnt)[t] = c.cnt;
        reinterpret_cast<float *>(ws + p.ws_amax)[t] = c.amax;
    }
}

// ---------------------------------------------------------------- k_scan (one workgroup)

__global__ void __launch_bounds__(1024)
k_scan(const Params p, uint8_t *__restrict__ blob, const uint8_t *__restrict__ ws) {
    __shared__ uint32_t scr[2][kMaxWaves][2];
    const uint32_t *cnt = reinterpret_cast<const uint32_t *>(ws + p.ws_cnt);
    const uint8_t *bits = blob + p.off_bits;
    uint64_t *row_ptr = reinterpret_cast<uint64_t *>(blob + p.off_row_ptr);
    uint64_t *pay_off = reinterpret_cast<uint64_t *>(blob + p.off_pay_off);
    const uint32_t tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, nw = blockDim.x >> 6;
    constexpr uint32_t kItems = 4;

    uint64_t carry_c = 0, carry_b = 0;
    uint32_t it = 0;
    for (uint64_t base = 0; base < p.tokens; base += (uint64_t)blockDim.x * kItems, ++it) {
        uint32_t c[kItems], y[kItems];
        uint32_t sc = 0, sy = 0;
#pragma unroll
        for (uint32_t k = 0; k < kItems; ++k) {
            const uint64_t t = base + (uint64_t)tid * kItems + k;
            c[k] = 0; y[k] = 0;
            if (t < p.tokens) { c[k] = cnt[t]; y[k] = row_bytes(p.hidden, bits[t]); }
            sc += c[k]; sy += y[k];
        }
        // inclusive scan inside the wave
        const uint32_t ic = wave_incl_scan_u32(sc), iy = wave_incl_scan_u32(sy);
        uint32_t (*s)[2] = scr[it & 1];
        if (lane == 63) { s[wv][0] = ic; s[wv][1] = iy; }
        __syncthreads();
        uint32_t bc = 0, by = 0, tc = 0, ty = 0;
        for (uint32_t w = 0; w < nw; ++w) {
            const uint32_t a = s[w][0], b = s[w][1];
            if (w < wv) { bc += a; by += b; }
            tc += a; ty += b;
        }
        uint64_t ec = carry_c + bc + ic - sc, ey = carry_b + by + iy - sy;
#pragma unroll
        for (uint32_t k = 0; k < kItems; ++k) {
            const uint64_t t = base + (uint64_t)tid * kItems + k;
            if (t < p.tokens) { row_ptr[t] = ec; pay_off[t] = ey; }
            ec += c[k]; ey += y[k];
        }
        carry_c += tc;
        carry_b += ty;
    }
    if (tid == 0) {
        row_ptr[p.tokens] = carry_c;
        pay_off[p.tokens] = carry_b;
        BlobHeader h;
        h.magic = kMagic; h.version = kVersion; h.dtype = p.dtype; h.tokens = p.tokens; h.hidden = p.hidden;
        h.tau_bits = __float_as_uint(p.tau); h.bit_mask = p.bit_mask; h.budget_bits = __float_as_uint(p.budget);
        h.mode = (uint32_t)p.mode;
        h.status = carry_c > p.outlier_capacity ? 3u : 0u;
        h.nnz = carry_c; h.payload_bytes = carry_b;
        h.off_bits = p.off_bits; h.off_scale = p.off_scale; h.off_pay_off = p.off_pay_off;
        h.off_row_ptr = p.off_row_ptr; h.off_payload = p.off_payload; h.off_out_col = p.off_out_col;
        h.off_out_val = p.off_out_val; h.payload_capacity = p.payload_capacity;
        h.outlier_capacity = p.outlier_capacity;
        *reinterpret_cast<BlobHeader *>(blob) = h;
    }
}

// ---------------------------------------------------------------- k_pack

template <int DT>
__global__ void __launch_bounds__(1024)
k_pack(const Params p, const uint16_t *__restrict__ in, uint8_t *__restrict__ blob, const uint8_t *__restrict__ ws) {
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t *lrow = lds;
    uint32_t *scratch = lds + p.runs * kRunLdsDw;
    const uint32_t t = blockIdx.x;
    const uint32_t run = threadIdx.x;

    const uint32_t width = blob[p.off_bits + t];
    const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
    const uint64_t rp0 = reinterpret_cast<const uint64_t *>(blob + p.off_row_ptr)[t];
    const uint64_t rp1 = reinterpret_cast<const uint64_t *>(blob + p.off_row_ptr)[t + 1];
    // the token's inlier absmax and outlier count are k_row_stats' results
    const float amax = reinterpret_cast<const float *>(ws + p.ws_amax)[t];
    const uint32_t cnt = reinterpret_cast<const uint32_t *>(ws + p.ws_cnt)[t];

    stage_row(reinterpret_cast<const uint4 *>(in + (size_t)t * p.hidden), p.pieces, p.runs, lrow);
    __syncthreads();

    uint32_t apk[16], omask = 0, amax_pk = 0;
    if (run < p.runs) split_run<false>(lrow + run * kRunLdsDw, p.thr_pk, apk, omask, amax_pk);
    const float r = amax >= kAmaxFloor ? level_count(width) / amax : 0.0f;

    // a width outside the plan's set would overrun the payload section: write nothing for it
    const bool width_ok = width >= 2 && width <= 8 && po + row_bytes(p.hidden, width) <= p.payload_capacity;
    if (run < p.runs && width_ok) {
        float af[32];
        widen_run<DT>(apk, af);
        uint32_t m[8];
        quantize_run(af, r, m);
        const uint32_t left = p.pieces - 4 * run;
        store_codes_any(width, m, lrow + run * kRunLdsDw, reinterpret_cast<uint32_t *>(blob + p.off_payload + po),
                        run, left < 4 ? left : 4);
    }
    // side stream: only tokens that fit entirely below the capacity are stored
    if (cnt > 0 && rp1 <= p.outlier_capacity && rp1 - rp0 == cnt) {
        emit_outliers(omask, lrow, run, reinterpret_cast<uint16_t *>(blob + p.off_out_col),
                      reinterpret_cast<uint16_t *>(blob + p.off_out_val), rp0, scratch + kScrScan);
    }
}

// ---------------------------------------------------------------- k_fused: one pass over the input
//
// Workgroup 1+t compresses token t; workgroup 0 (dispatched first) is the scan workgroup.
//
//   compute workgroup:  load the row (each lane its run, straight into registers), split, choose
//       the width, publish agg[t] = (payload words, outlier count), pack the codes into
//       registers, wait for pref[t], store.
//   scan workgroup:  streams over the tokens in order.  Each round it reads a window of agg words
//       starting at the first unpublished token, takes the longest run of valid ones, scans it on
//       top of a running total and publishes pref[t] = exclusive prefix; it also writes row_ptr /
//       pay_off and, at the end, the blob header.  pref[t] depends on tokens before t only, all of
//       which were dispatched before t.
//
// agg and pref words: bit 62 = valid, bit 63 = error, bits 61..32 words, bits 31..0 count; both
// sums stay below 2^30 / 2^32 because tokens*hidden < 2^32.  They are written and read with
// device-coherent relaxed atomics (the values are self-contained, nothing else is ordered by
// them).  Two generations of both arrays alternate between calls: a call fills one and zeroes
// the other, so no clearing pass is needed.  Every wait is bounded by p.spin_limit.
constexpr uint64_t kWordValid = 1ull << 62, kWordError = 1ull << 63;
constexpr int kScanItems = 8;  // tokens per thread and round in the scan workgroup

enum { kCtlGen = 0, kCtlError = 1 };

__device__ __forceinline__ uint64_t word_load(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void word_store(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t wait_word(const uint64_t *p, uint32_t spin_limit) {
    uint64_t v = word_load(p);
    uint32_t spins = 0;
    while (!(v & kWordValid) && spins < spin_limit) {
        __builtin_amdgcn_s_sleep(1);
        v = word_load(p);
        ++spins;
    }
    return v;
}

__device__ __forceinline__ void write_header(const Params &p, uint8_t *blob, uint64_t nnz, uint64_t payload_bytes,
                                             uint32_t status) {
    BlobHeader h;
    h.magic = kMagic; h.version = kVersion; h.dtype = p.dtype; h.tokens = p.tokens; h.hidden = p.hidden;
    h.tau_bits = __float_as_uint(p.tau); h.bit_mask = p.bit_mask; h.budget_bits = __float_as_uint(p.budget);
    h.mode = (uint32_t)p.mode;
    h.status = status;
    h.nnz = nnz; h.payload_bytes = payload_bytes;
    h.off_bits = p.off_bits; h.off_scale = p.off_scale; h.off_pay_off = p.off_pay_off;
    h.off_row_ptr = p.off_row_ptr; h.off_payload = p.off_payload; h.off_out_col = p.off_out_col;
    h.off_out_val = p.off_out_val; h.payload_capacity = p.payload_capacity;
    h.outlier_capacity = p.outlier_capacity;
    *reinterpret_cast<BlobHeader *>(blob) = h;
}

template <int B>
__device__ __forceinline__ void pack_into(const uint32_t (&m)[8], const uint32_t (&w)[16], uint32_t (&out)[8]) {
    uint32_t o[B];
    pack_regs<B>(m, w, o);
#pragma unroll
    for (int k = 0; k < B; ++k) out[k] = o[k];
}

// What a compute workgroup keeps of a token between publishing it and storing it.
struct Pending {
    uint32_t out[8];   // packed codes of the lane's run (first `width` dwords)
    uint32_t omask;    // the lane's outlier flags
    uint32_t loff;     // outliers of the token in lanes before this one
};

__device__ __forceinline__ void store_pending(const Params &p, uint8_t *blob, uint8_t *ws, const Pending &pd,
                                              uint32_t t, uint32_t width, uint32_t cnt, const uint32_t *slot,
                                              uint64_t pv, uint32_t run) {
    const uint64_t *pref = reinterpret_cast<const uint64_t *>(ws + p.ws_pref);
    (void)pref;
    bool ok = (pv & kWordValid) && !(pv & kWordError);
    const uint32_t ew = (uint32_t)(pv >> 32) & 0x3FFFFFFFu, ec = (uint32_t)pv;
    const uint32_t words = row_bytes(p.hidden, width) >> 2;
    if ((uint64_t)ew + words > (p.payload_capacity >> 2)) ok = false;  // never store outside the blob
    if (!ok) {
        if (threadIdx.x == 0) {
            uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
            __hip_atomic_fetch_or(ctrl + kCtlError, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // the header may already be final: make the blob unreadable
            __hip_atomic_store(reinterpret_cast<uint32_t *>(blob), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }
    if (run < p.runs) {
        const uint32_t left = p.pieces - 4 * run;
        const uint32_t nd = left >= 4 ? width : ((left * width + 3u) >> 2);
        uint32_t *dst = reinterpret_cast<uint32_t *>(blob + p.off_payload) + ew + run * width;
#pragma unroll
        for (uint32_t k = 0; k < 8; ++k)
            if (k < nd) dst[k] = pd.out[k];
        if (pd.omask && (uint64_t)ec + cnt <= p.outlier_capacity) {
            uint16_t *col = reinterpret_cast<uint16_t *>(blob + p.off_out_col);
            uint16_t *val = reinterpret_cast<uint16_t *>(blob + p.off_out_val);
            uint64_t pos = (uint64_t)ec + pd.loff;
            uint32_t ev = pd.omask & 0xFFFFu, od = pd.omask >> 16;
            while (ev | od) {
                const uint32_t je = ev ? 2u * (uint32_t)__builtin_ctz(ev) : 64u;
                const uint32_t jo = od ? 2u * (uint32_t)__builtin_ctz(od) + 1u : 64u;
                uint32_t j;
                if (je < jo) { j = je; ev &= ev - 1u; } else { j = jo; od &= od - 1u; }
                col[pos] = (uint16_t)(run * kRun + j);
                val[pos] = slot_raw(slot, run, j);
                ++pos;
            }
        }
    }
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    uint32_t n;
    n = dpp<kDppQuadXor1>(v);   v = n < v ? n : v;
    n = dpp<kDppQuadXor2>(v);   v = n < v ? n : v;
    n = dpp<kDppHalfMirror>(v); v = n < v ? n : v;
    n = dpp<kDppRowMirror>(v);  v = n < v ? n : v;
    const uint32_t a = lane_value(v, 0), b = lane_value(v, 16), c = lane_value(v, 32), d = lane_value(v, 48);
    const uint32_t ab = a < b ? a : b, cd = c < d ? c : d;
    return ab < cd ? ab : cd;
}

__device__ __forceinline__ void scan_stream(const Params &p, uint8_t *blob, uint8_t *ws, uint32_t gen, uint32_t *scr) {
    const uint64_t *agg = reinterpret_cast<const uint64_t *>(ws + p.ws_agg) + (size_t)gen * p.tokens;
    uint64_t *pref = reinterpret_cast<uint64_t *>(ws + p.ws_pref) + (size_t)gen * p.tokens;
    uint64_t *pref_next = reinterpret_cast<uint64_t *>(ws + p.ws_pref) + (size_t)(1u - gen) * p.tokens;
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    uint64_t *row_ptr = reinterpret_cast<uint64_t *>(blob + p.off_row_ptr);
    uint64_t *pay_off = reinterpret_cast<uint64_t *>(blob + p.off_pay_off);
    const uint32_t tid = threadIdx.x, wv = tid >> 6, nw = blockDim.x >> 6;
    const uint32_t window = blockDim.x * kScanItems;

    uint64_t carry_c = 0, carry_w = 0, start = 0;
    uint32_t failed = 0, it = 0, idle = 0;
    while (start < p.tokens) {
        uint64_t v[kScanItems];
        uint32_t first_missing = window;
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            const uint64_t t = start + (uint64_t)tid * kScanItems + k;
            v[k] = 0;
            if (t < p.tokens) v[k] = word_load(agg + t);
        }
#pragma unroll
        for (int k = kScanItems - 1; k >= 0; --k)
            if (!(v[k] & kWordValid)) first_missing = tid * kScanItems + k;
        // length of the run of valid words at the front of the window
        uint32_t *s4 = scr + (it & 1) * 4 * kMaxWaves;
        ++it;
        uint32_t n = wave_min_u32(first_missing);
        if (nw > 1) {
            if ((tid & 63) == 0) s4[4 * wv + 3] = n;
            __syncthreads();
            for (uint32_t w = 0; w < nw; ++w) { const uint32_t x = s4[4 * w + 3]; n = x < n ? x : n; }
        }
        const uint64_t remaining = p.tokens - start;
        if (n > remaining) n = (uint32_t)remaining;
        if (n == 0) {
            if (++idle > p.spin_limit) { failed = 1; n = remaining < window ? (uint32_t)remaining : window; }
            else { __builtin_amdgcn_s_sleep(1); continue; }
        }
        idle = 0;
        uint32_t sc = 0, sw = 0;
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            if (tid * kScanItems + k >= n || !(v[k] & kWordValid)) v[k] = 0;
            sc += (uint32_t)v[k];
            sw += (uint32_t)(v[k] >> 32) & 0x3FFFFFFFu;
        }
        const uint32_t ic = wave_incl_scan_u32(sc), iw = wave_incl_scan_u32(sw);
        uint32_t bc = 0, bw = 0, tc = ic, tw = iw;
        if (nw > 1) {
            uint32_t *s4b = scr + (it & 1) * 4 * kMaxWaves;
            ++it;
            if ((tid & 63) == 63) { s4b[4 * wv] = ic; s4b[4 * wv + 1] = iw; }
            __syncthreads();
            tc = 0; tw = 0;
            for (uint32_t w = 0; w < nw; ++w) {
                const uint32_t a = s4b[4 * w], b = s4b[4 * w + 1];
                if (w < wv) { bc += a; bw += b; }
                tc += a; tw += b;
            }
        } else {
            tc = lane_value(ic, 63); tw = lane_value(iw, 63);
        }
        uint64_t ec = carry_c + bc + ic - sc, ew = carry_w + bw + iw - sw;
        const uint64_t flags = kWordValid | (failed ? kWordError : 0ull);
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            if (tid * kScanItems + k < n) {
                const uint64_t t = start + (uint64_t)tid * kScanItems + k;
                word_store(pref + t, flags | ((ew & 0x3FFFFFFFull) << 32) | (ec & 0xFFFFFFFFull));
                pref_next[t] = 0;
                row_ptr[t] = ec;
                pay_off[t] = ew << 2;
            }
            ec += (uint32_t)v[k];
            ew += (uint32_t)(v[k] >> 32) & 0x3FFFFFFFu;
        }
        carry_c += tc;
        carry_w += tw;
        start += n;
    }
    if (tid == 0) {
        row_ptr[p.tokens] = carry_c;
        pay_off[p.tokens] = carry_w << 2;
        const uint32_t err = failed | __hip_atomic_load(ctrl + kCtlError, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        write_header(p, blob, carry_c, carry_w << 2, err ? 6u : (carry_c > p.outlier_capacity ? 3u : 0u));
        __hip_atomic_store(ctrl + kCtlError, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(ctrl + kCtlGen, gen ^ 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int DT>
__global__ void __launch_bounds__(1024)
k_fused(const Params p, const uint16_t *__restrict__ in, uint8_t *__restrict__ blob, uint8_t *__restrict__ ws) {
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t *slot = lds;
    uint32_t *scratch = lds + p.runs * 16;
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint32_t gen = ctrl[kCtlGen] & 1u;
    if (blockIdx.x == 0) {
        scan_stream(p, blob, ws, gen, scratch);
        return;
    }
    const uint32_t t = blockIdx.x - 1;
    uint64_t *agg = reinterpret_cast<uint64_t *>(ws + p.ws_agg) + (size_t)gen * p.tokens;
    uint64_t *agg_next = reinterpret_cast<uint64_t *>(ws + p.ws_agg) + (size_t)(1u - gen) * p.tokens;
    const uint64_t *pref = reinterpret_cast<const uint64_t *>(ws + p.ws_pref) + (size_t)gen * p.tokens;
    const uint32_t run = threadIdx.x;
    const bool owns = run < p.runs;
    const uint32_t left = owns ? p.pieces - 4 * run : 0;
    clear_reduce_areas(scratch);
    __syncthreads();

    uint32_t apk[16], omask = 0, amax_pk = 0;
    if (owns) {
        uint32_t w[16];
        const uint4 *src = reinterpret_cast<const uint4 *>(in + (size_t)t * p.hidden) + 4 * run;
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            uint4 q = make_uint4(0, 0, 0, 0);
            if (k < left) q = src[k];
            w[4 * k] = q.x; w[4 * k + 1] = q.y; w[4 * k + 2] = q.z; w[4 * k + 3] = q.w;
        }
        slot_write(slot, run, w);
        split_regs<true>(w, p.thr_pk, apk, omask, amax_pk);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) apk[i] = 0;
    }
    uint32_t m[8];
    const Choice c = choose_width<DT>(p, apk, omask, amax_pk, scratch, m);
    if (threadIdx.x == 0) {
        const uint32_t words = row_bytes(p.hidden, c.width) >> 2;
        word_store(agg + t, kWordValid | ((uint64_t)words << 32) | c.cnt);
        agg_next[t] = 0;
        blob[p.off_bits + t] = (uint8_t)c.width;
        reinterpret_cast<float *>(blob + p.off_scale)[t] = scale_of(c.amax, c.width);
    }
    Pending pd;
    pd.omask = omask;
    pd.loff = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) pd.out[k] = 0;
    if (owns) {
        uint32_t wr[16];
        slot_read(slot, run, wr);
        switch (c.width) {
            case 2: pack_into<2>(m, wr, pd.out); break;
            case 3: pack_into<3>(m, wr, pd.out); break;
            case 4: pack_into<4>(m, wr, pd.out); break;
            case 5: pack_into<5>(m, wr, pd.out); break;
            case 6: pack_into<6>(m, wr, pd.out); break;
            case 7: pack_into<7>(m, wr, pd.out); break;
            default: pack_into<8>(m, wr, pd.out); break;
        }
    }
    if (c.cnt > 0) pd.loff = block_excl_scan((uint32_t)__builtin_popcount(omask), scratch + kScrScan);
    // wave 0 waits for the token's position and hands it to the others
    uint32_t *bc = scratch + kScrBcast;
    if (threadIdx.x < 64) {
        const uint64_t pv = wait_word(pref + t, p.spin_limit);
        if (threadIdx.x == 0) { bc[0] = (uint32_t)pv; bc[1] = (uint32_t)(pv >> 32); }
    }
    __syncthreads();
    const uint64_t pv = ((uint64_t)bc[1] << 32) | bc[0];
    store_pending(p, blob, ws, pd, t, c.width, c.cnt, slot, pv, run);
}

// ---------------------------------------------------------------- k_unpack

template <int DT, int B>
__device__ __forceinline__ void load_and_unpack(const uint32_t *src_row, uint32_t run, uint32_t valid_pieces, float s,
                                                uint32_t *lrun) {
    uint32_t d[B];
    const uint32_t *src = src_row + run * B;
    if (valid_pieces >= 4) {
#pragma unroll
        for (int k = 0; k < B; ++k) d[k] = src[k];
    } else {
        const uint32_t nd = (valid_pieces * B + 3u) >> 2;
#pragma unroll
        for (int k = 0; k < B; ++k) d[k] = (uint32_t)k < nd ? src[k] : 0u;
    }
    uint32_t o[16];
    unpack_run<DT, B>(d, s, o);
#pragma unroll
    for (int k = 0; k < 4; ++k)
        *reinterpret_cast<uint4 *>(lrun + 4 * k) = make_uint4(o[4 * k], o[4 * k + 1], o[4 * k + 2], o[4 * k + 3]);
}

template <int DT>
__global__ void __launch_bounds__(1024)
k_unpack(const Params p, const uint8_t *__restrict__ blob, uint16_t *__restrict__ out) {
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t *lrow = lds;
    const uint32_t t = blockIdx.x;
    const uint32_t run = threadIdx.x;

    // the blob must be this plan's and must have been completed without error
    const BlobHeader *h = reinterpret_cast<const BlobHeader *>(blob);
    if (h->magic != kMagic || h->version != kVersion || h->status != 0 || h->tokens != p.tokens ||
        h->hidden != p.hidden || h->dtype != p.dtype || h->off_payload != p.off_payload ||
        h->off_out_col != p.off_out_col || h->off_out_val != p.off_out_val)
        return;

    const uint32_t width = blob[p.off_bits + t];
    const float s = reinterpret_cast<const float *>(blob + p.off_scale)[t];
    const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
    const uint64_t rp0 = reinterpret_cast<const uint64_t *>(blob + p.off_row_ptr)[t];
    const uint64_t rp1 = reinterpret_cast<const uint64_t *>(blob + p.off_row_ptr)[t + 1];
    // a damaged token is skipped rather than read out of bounds
    if (width < 2 || width > 8 || (po & 3u) || po + row_bytes(p.hidden, width) > p.payload_capacity ||
        rp0 > rp1 || rp1 > p.outlier_capacity)
        return;

    if (run < p.runs) {
        const uint32_t left = p.pieces - 4 * run;
        const uint32_t vp = left < 4 ? left : 4;
        const uint32_t *src_row = reinterpret_cast<const uint32_t *>(blob + p.off_payload + po);
        uint32_t *lrun = lrow + run * kRunLdsDw;
        switch (width) {
            case 2: load_and_unpack<DT, 2>(src_row, run, vp, s, lrun); break;
            case 3: load_and_unpack<DT, 3>(src_row, run, vp, s, lrun); break;
            case 4: load_and_unpack<DT, 4>(src_row, run, vp, s, lrun); break;
            case 5: load_and_unpack<DT, 5>(src_row, run, vp, s, lrun); break;
            case 6: load_and_unpack<DT, 6>(src_row, run, vp, s, lrun); break;
            case 7: load_and_unpack<DT, 7>(src_row, run, vp, s, lrun); break;
            default: load_and_unpack<DT, 8>(src_row, run, vp, s, lrun); break;
        }
    }
    __syncthreads();
    // + T_above: outliers overwrite their slots with the stored bits
    {
        const uint16_t *col = reinterpret_cast<const uint16_t *>(blob + p.off_out_col);
        const uint16_t *val = reinterpret_cast<const uint16_t *>(blob + p.off_out_val);
        uint16_t *lrow16 = reinterpret_cast<uint16_t *>(lrow);
        for (uint64_t k = rp0 + threadIdx.x; k < rp1; k += blockDim.x) {
            const uint32_t c = col[k];
            if (c < p.hidden) lrow16[(c >> 5) * (2 * kRunLdsDw) + (c & 31u)] = val[k];
        }
    }
    __syncthreads();
    uint4 *dst = reinterpret_cast<uint4 *>(out + (size_t)t * p.hidden);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t q = threadIdx.x + k * blockDim.x;
        if (q < p.pieces) dst[q] = *reinterpret_cast<const uint4 *>(lrow + (q >> 2) * kRunLdsDw + (q & 3) * 4);
    }
}

// ---------------------------------------------------------------- launchers

static hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

int prepare_kernels() {
    const int big = (int)((kMaxHidden / kRun) * kRunLdsDw * 4 + kScratchDw * 4);
    hipError_t e;
#define TSQ_RAISE(k)                                                                                     \
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, big); \
    if (e != hipSuccess) return (int)e;
    TSQ_RAISE(k_row_stats<kF16>)
    TSQ_RAISE(k_row_stats<kBF16>)
    TSQ_RAISE(k_pack<kF16>)
    TSQ_RAISE(k_pack<kBF16>)
    TSQ_RAISE(k_fused<kF16>)
    TSQ_RAISE(k_fused<kBF16>)
    TSQ_RAISE(k_unpack<kF16>)
    TSQ_RAISE(k_unpack<kBF16>)
#undef TSQ_RAISE
    return 0;
}

int launch_row_stats(const Params &p, const Geometry &g, const void *d_in, void *d_blob, void *d_ws, void *stream) {
    const dim3 grid(p.tokens), block(g.block);
    if (p.dtype == kF16)
        hipLaunchKernelGGL(k_row_stats<kF16>, grid, block, g.lds_bytes, as_stream(stream), p,
                           static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                           static_cast<uint8_t *>(d_ws));
    else
        hipLaunchKernelGGL(k_row_stats<kBF16>, grid, block, g.lds_bytes, as_stream(stream), p,
                           static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                           static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

int launch_scan(const Params &p, void *d_blob, void *d_ws, void *stream) {
    const uint32_t need = (p.tokens + 3) / 4;
    uint32_t block = 64;
    while (block < 1024 && block < need) block *= 2;
    hipLaunchKernelGGL(k_scan, dim3(1), dim3(block), 0, as_stream(stream), p, static_cast<uint8_t *>(d_blob),
                       static_cast<const uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

int launch_pack(const Params &p, const Geometry &g, const void *d_in, void *d_blob, void *d_ws, void *stream) {
    const dim3 grid(p.tokens), block(g.block);
    if (p.dtype == kF16)
        hipLaunchKernelGGL(k_pack<kF16>, grid, block, g.lds_bytes, as_stream(stream), p,
                           static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                           static_cast<const uint8_t *>(d_ws));
    else
        hipLaunchKernelGGL(k_pack<kBF16>, grid, block, g.lds_bytes, as_stream(stream), p,
                           static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                           static_cast<const uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

int launch_unpack(const Params &p, const Geometry &g, const void *d_blob, void *d_out, void *stream) {
    const dim3 grid(p.tokens), block(g.block);
    if (p.dtype == kF16)
        hipLaunchKernelGGL(k_unpack<kF16>, grid, block, g.lds_bytes, as_stream(stream), p,
                           static_cast<const uint8_t *>(d_blob), static_cast<uint16_t *>(d_out));
    else
        hipLaunchKernelGGL(k_unpack<kBF16>, grid, block, g.lds_bytes, as_stream(stream), p,
                           static_cast<const uint8_t *>(d_blob), static_cast<uint16_t *>(d_out));
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------- workspace reset

__global__ void k_ws_reset(const Params p, uint8_t *__restrict__ ws) {
    uint64_t *agg = reinterpret_cast<uint64_t *>(ws + p.ws_agg);
    uint64_t *pref = reinterpret_cast<uint64_t *>(ws + p.ws_pref);
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 2ull * p.tokens) { agg[i] = 0; pref[i] = 0; }
    if (i < 64) ctrl[i] = 0;
}

int launch_ws_reset(const Params &p, void *d_ws, void *stream) {
    const uint64_t n = 2ull * p.tokens > 64 ? 2ull * p.tokens : 64;
    hipLaunchKernelGGL(k_ws_reset, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, as_stream(stream), p,
                       static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

int launch_fused(const Params &p, const Geometry &g, const void *d_in, void *d_blob, void *d_ws, void *stream) {
    const dim3 grid(p.tokens + 1), block(g.block);
    if (p.dtype == kF16)
        hipLaunchKernelGGL(k_fused<kF16>, grid, block, g.lds_fused_bytes, as_stream(stream), p,
                           static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                           static_cast<uint8_t *>(d_ws));
    else
        hipLaunchKernelGGL(k_fused<kBF16>, grid, block, g.lds_fused_bytes, as_stream(stream), p,
                           static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                           static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

}  // namespace tsq
