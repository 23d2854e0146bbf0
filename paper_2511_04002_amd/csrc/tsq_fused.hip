// Single-pass compress kernel (gfx950): Eq. (ts), Algorithm 1, Eq. (Proposed), bit packing and
// CSR emission with ONE read of the input.
//
// A persistent grid of G workgroups, all resident at once; workgroup g compresses tokens
// g, g + G, g + 2G, ...  The tokens [k*G, (k+1)*G) form "generation" k: every workgroup is
// working on the same generation at roughly the same time.
//
// Placement of the variable-length outputs (payload words, CSR entries) needs the exclusive
// prefix over all earlier tokens.  Each workgroup publishes its token's (words, outliers) pair
// in a table slot; a workgroup finds the prefix of its token by reading the G pairs of the
// token's generation (earlier workgroup ids give the prefix inside the generation, all of them
// the generation's total, which is carried forward as a running base).  Nobody scans on behalf
// of the others, so there is no serial chain across workgroups: one hop from publish to use.
//
// To keep that hop off the critical path, a token is stored one iteration late: iteration i
// computes token i (codes stay in registers, outliers in an LDS stash), publishes it, and then
// stores token i-1, whose generation was published by everybody about one iteration ago.  The
// input row of iteration i+1 is fetched into registers at the top of iteration i.
//
// Table words are 32 bit (2-bit generation tag, payload words, outlier count).  There are four
// slots per workgroup (generation & 3): a workgroup can be at most two generations ahead of the
// slowest reader of a slot.  Two banks of the table alternate between calls; a call
// clears the bank of the next call, so no separate clearing pass is needed.  Words are written
// and read with relaxed device-scope atomics; they carry their own validity, nothing else is
// ordered through them.  Every wait is bounded by p.spin_limit; an expired wait marks the blob
// as failed (TSQ_ERR_INTERNAL) instead of hanging.
#include <hip/hip_runtime.h>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

enum { kCtlBank = 0, kCtlError = 1 };

// Table words (32 bit): bits 31..30 = tag of the generation (generation % 3 + 1; 0 = empty),
// bits 29..16 = payload words of the token (<= 8192), bits 15..0 = its outliers (<= 32768).
// A slot (generation & 3) is reused every fourth generation; three successive users of a slot
// have three different tags, and no reader is ever more than two generations behind a writer.
__device__ __forceinline__ uint32_t word_load(const uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void word_store(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t gen_tag(uint32_t gen) { return gen % 3u + 1u; }

template <int B>
__device__ __forceinline__ void pack_into(const uint32_t (&m)[8], const uint32_t (&w)[16], uint32_t (&out)[8]) {
    uint32_t o[B];
    pack_regs<B>(m, w, o);
#pragma unroll
    for (int k = 0; k < B; ++k) out[k] = o[k];
}

// B consecutive dwords to a 4-byte aligned address, in as few store instructions as possible.
struct __attribute__((packed, aligned(4))) Dw4 { uint32_t a, b, c, d; };
struct __attribute__((packed, aligned(4))) Dw2 { uint32_t a, b; };
template <int B>
__device__ __forceinline__ void store_dwords(uint32_t *dst, const uint32_t (&o)[8]) {
    int k = 0;
    if (B - k >= 4) { *reinterpret_cast<Dw4 *>(dst + k) = Dw4{o[k], o[k + 1], o[k + 2], o[k + 3]}; k += 4; }
    if (B - k >= 4) { *reinterpret_cast<Dw4 *>(dst + k) = Dw4{o[k], o[k + 1], o[k + 2], o[k + 3]}; k += 4; }
    if (B - k >= 2) { *reinterpret_cast<Dw2 *>(dst + k) = Dw2{o[k], o[k + 1]}; k += 2; }
    if (B - k >= 1) { dst[k] = o[k]; }
}

// ---- placement: prefix of this workgroup inside a generation, and the generation's totals ----
struct GenSums {
    uint32_t pre_w, pre_c;   // payload words / outliers of the generation's tokens before ours
    uint32_t tot_w, tot_c;   // of all tokens of the generation
    uint32_t bad;            // a wait expired
};
constexpr int kEarly = 4;    // table words per thread that are requested an iteration's work early

template <int NW>
__device__ __forceinline__ void request_generation(const uint32_t *slots, uint32_t n, uint32_t (&e)[kEarly]) {
#pragma unroll
    for (int k = 0; k < kEarly; ++k) {
        const uint32_t j = threadIdx.x + (uint32_t)k * 64u * NW;
        e[k] = 0;
        if (j < n) e[k] = word_load(slots + j);
    }
}

// e: the words request_generation asked for (re-read here while they are not valid yet);
// words beyond kEarly per thread are read here.  area: 5*kMaxWaves dwords of LDS.
// All threads of the block call this (one barrier).
template <int NW>
__device__ __forceinline__ GenSums resolve_generation(const uint32_t *slots, uint32_t n, uint32_t wg, uint32_t tag,
                                                      uint32_t spin_limit, const uint32_t (&e)[kEarly],
                                                      uint32_t *area) {
    constexpr uint32_t kThreads = 64 * NW;
#ifdef X_NORESOLVE
    { GenSums z; z.pre_w = z.pre_c = z.tot_w = z.tot_c = z.bad = 0; return z; }
#endif
    uint32_t pw = 0, pc = 0, tw = 0, tc = 0, bad = 0;
    auto take = [&](uint32_t j, uint32_t v) {
        uint32_t spins = 0;
        while ((v >> 30) != tag && spins < spin_limit) {
            __builtin_amdgcn_s_sleep(2);
            v = word_load(slots + j);
            ++spins;
        }
        if ((v >> 30) != tag) { bad = 1; v = 0; }
        const uint32_t w = (v >> 16) & 0x3FFFu, c = v & 0xFFFFu;
        tw += w;
        tc += c;
        if (j < wg) { pw += w; pc += c; }
    };
#pragma unroll
    for (int k = 0; k < kEarly; ++k) {
        const uint32_t j = threadIdx.x + (uint32_t)k * kThreads;
        if (j < n) take(j, e[k]);
    }
    for (uint32_t j = threadIdx.x + kEarly * kThreads; j < n; j += kThreads) take(j, word_load(slots + j));

    pw = wave_sum_u32(pw); pc = wave_sum_u32(pc); tw = wave_sum_u32(tw); tc = wave_sum_u32(tc);
    bad = __builtin_amdgcn_ballot_w64(bad != 0) != 0 ? 1u : 0u;
    GenSums g;
    if (NW == 1) {
        g.pre_w = pw; g.pre_c = pc; g.tot_w = tw; g.tot_c = tc; g.bad = bad;
        return g;
    }
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) {
        area[0 * kMaxWaves + wv] = pw; area[1 * kMaxWaves + wv] = pc; area[2 * kMaxWaves + wv] = tw;
        area[3 * kMaxWaves + wv] = tc; area[4 * kMaxWaves + wv] = bad;
    }
    __syncthreads();
    uint32_t s[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        uint32_t a = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) a += area[k * kMaxWaves + w];
        s[k] = a;
    }
    g.pre_w = uniform(s[0]); g.pre_c = uniform(s[1]); g.tot_w = uniform(s[2]); g.tot_c = uniform(s[3]);
    g.bad = uniform(s[4]);
    return g;
}

// What a workgroup keeps of a token between computing it and storing it.
struct Pending {
    uint32_t out[8];   // packed codes of the lane's run (first `width` dwords)
    uint32_t width, cnt, token, gen;
};

// LDS map (dynamic): row: runs*kRunLdsDw | ring: 4 reduce areas | two resolve areas | two stashes
constexpr uint32_t kLdsRing = 4 * 2 * kMaxWaves, kLdsResolve = 5 * kMaxWaves;
static_assert(kFusedScratchDw == kLdsRing + 2 * kLdsResolve + 2 * kStashCap, "LDS map of the fused kernel");

template <int DT, int NW>
__global__ void __launch_bounds__(64 * NW, 4)
k_fused(const Params p, const uint16_t *__restrict__ in, uint8_t *__restrict__ blob, uint8_t *__restrict__ ws) {
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr uint32_t kThreads = 64 * NW;
    uint32_t *lrow = lds;
    uint32_t *ring = lds + p.runs * kRunLdsDw;
    uint32_t *areas = ring + kLdsRing;
    uint32_t *stashes = areas + 2 * kLdsResolve;            // 2 x kStashCap dwords: col << 16 | raw value
    const uint32_t tid = threadIdx.x, run = tid;
    const uint32_t wg = blockIdx.x, G = gridDim.x;
    const bool owns = run < p.runs;
    const uint32_t left = owns ? p.pieces - 4 * run : 0;    // 16-byte pieces of the lane's run inside the row

    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint32_t bank = ctrl[kCtlBank] & 1u;
    uint32_t *table = reinterpret_cast<uint32_t *>(ws + p.ws_agg) + (size_t)bank * 4 * kFusedGridCap;
    uint32_t *table_next = reinterpret_cast<uint32_t *>(ws + p.ws_agg) + (size_t)(1u - bank) * 4 * kFusedGridCap;
    if (tid < 4) table_next[tid * kFusedGridCap + wg] = 0;

    uint8_t *bits = blob + p.off_bits;
    float *scale = reinterpret_cast<float *>(blob + p.off_scale);
    uint64_t *pay_off = reinterpret_cast<uint64_t *>(blob + p.off_pay_off);
    uint64_t *row_ptr = reinterpret_cast<uint64_t *>(blob + p.off_row_ptr);
    uint32_t *payload = reinterpret_cast<uint32_t *>(blob + p.off_payload);
    uint16_t *out_col = reinterpret_cast<uint16_t *>(blob + p.off_out_col);
    uint16_t *out_val = reinterpret_cast<uint16_t *>(blob + p.off_out_val);

    // the row of the next iteration on its way HBM -> registers -> LDS (each wave its own part)
    uint4 pre[4];
    auto fetch_row = [&](uint32_t t) {
        fetch_row_part(reinterpret_cast<const uint4 *>(in + (size_t)t * p.hidden), p.pieces, pre);
    };
    auto write_row = [&]() { write_row_part(lrow, p.runs, pre); };

    uint32_t base_w = 0, base_c = 0;     // totals of all generations already resolved
    uint32_t failed = 0, turn = 0;
    Pending pd;
    bool have_pending = false;
    pd.width = 8; pd.cnt = 0; pd.token = 0; pd.gen = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) pd.out[k] = 0;

    auto gen_size = [&](uint32_t gen) { return p.tokens - gen * G < G ? p.tokens - gen * G : G; };

    // stores a token whose generation sums are known: payload from registers, outliers from its stash
    auto store_token = [&](const Pending &q, const GenSums &g, bool from_stash) {
        const uint32_t ew = base_w + g.pre_w, ec = base_c + g.pre_c;
        if (tid == 0) {
            pay_off[q.token] = (uint64_t)ew << 2;
            row_ptr[q.token] = ec;
        }
        if (owns) {
            uint32_t *dst = payload + ew + run * q.width;
            if (left >= 4) {
                switch (q.width) {
                    case 2: store_dwords<2>(dst, q.out); break;
                    case 3: store_dwords<3>(dst, q.out); break;
                    case 4: store_dwords<4>(dst, q.out); break;
                    case 5: store_dwords<5>(dst, q.out); break;
                    case 6: store_dwords<6>(dst, q.out); break;
                    case 7: store_dwords<7>(dst, q.out); break;
                    default: store_dwords<8>(dst, q.out); break;
                }
            } else {
                const uint32_t nd = (left * q.width + 3u) >> 2;
#pragma unroll
                for (uint32_t k = 0; k < 8; ++k)
                    if (k < nd) dst[k] = q.out[k];
            }
        }
        if (from_stash && q.cnt > 0 && (uint64_t)ec + q.cnt <= p.outlier_capacity) {
            const uint32_t *stash = stashes + (q.gen & 1u) * kStashCap;
            for (uint32_t k = tid; k < q.cnt; k += kThreads) {
                const uint32_t e = stash[k];
                out_col[(size_t)ec + k] = (uint16_t)(e >> 16);
                out_val[(size_t)ec + k] = (uint16_t)e;
            }
        }
    };

    uint32_t t = wg;
    fetch_row(t);
    write_row();

    uint32_t it = 0;
    for (; t < p.tokens; ++it, t += G) {
        const uint32_t tn = t + G;
        // the table words of the pending token's generation: asked for now, used after the width search
        uint32_t early[kEarly];
#ifndef X_NORESOLVE
        if (have_pending)
            request_generation<NW>(table + (pd.gen & 3u) * kFusedGridCap, gen_size(pd.gen), early);
#endif

        // ---- Eq. (ts) and Algorithm 1 for token t
        Mags<DT> mg;
        uint32_t omask = 0, amax_bits = 0;
        split_run<DT, true>(lrow + (owns ? run : 0u) * kRunLdsDw, p.thr_pk, mg, omask, amax_bits);
        if (!owns) omask = 0;
        uint32_t m[8], cnt_before;
        const Choice c = choose_width<DT, NW>(p, mg, omask, amax_bits, owns, ring, turn, m, cnt_before);
        const uint32_t words = row_bytes(p.hidden, c.width) >> 2;
        if (tid == 0) {
            word_store(table + (it & 3u) * kFusedGridCap + wg, (gen_tag(it) << 30) | (words << 16) | c.cnt);
            bits[t] = (uint8_t)c.width;
            scale[t] = scale_of(c.amax, c.width);
        }
        // the next row starts its way from HBM now that the registers of the width search are free
        if (tn < p.tokens) fetch_row(tn);

        // ---- codes of the lane's run at the chosen width
        Pending cur;
        cur.width = c.width; cur.cnt = c.cnt; cur.token = t; cur.gen = it;
#pragma unroll
        for (int k = 0; k < 8; ++k) cur.out[k] = 0;
        if (owns) {
            uint32_t wr[16];
            load_run_padded(lrow + run * kRunLdsDw, wr);
            switch (c.width) {
                case 2: pack_into<2>(m, wr, cur.out); break;
                case 3: pack_into<3>(m, wr, cur.out); break;
                case 4: pack_into<4>(m, wr, cur.out); break;
                case 5: pack_into<5>(m, wr, cur.out); break;
                case 6: pack_into<6>(m, wr, cur.out); break;
                case 7: pack_into<7>(m, wr, cur.out); break;
                default: pack_into<8>(m, wr, cur.out); break;
            }
        }

        // ---- store the token of the previous iteration
        if (have_pending) {
#ifdef X_NORESOLVE
            GenSums g; g.pre_w = g.pre_c = g.tot_w = g.tot_c = g.bad = 0;
#else
            const GenSums g = resolve_generation<NW>(table + (pd.gen & 3u) * kFusedGridCap, gen_size(pd.gen), wg,
                                                     gen_tag(pd.gen), p.spin_limit, early,
                                                     areas + (pd.gen & 1u) * kLdsResolve);
#endif
            failed |= g.bad;
#ifndef X_NOSTORE
            if (!g.bad) store_token(pd, g, true);
#endif
            base_w += g.tot_w;
            base_c += g.tot_c;
            have_pending = false;
        }

        // ---- T_above of token t: into this generation's stash in column order, or straight out if
        //      it is too long for the stash
        bool placed = false;
        if (c.cnt > 0) {
            const uint32_t nl = (uint32_t)__builtin_popcount(omask);
            const uint32_t loff = cnt_before + wave_incl_scan_u32(nl) - nl;
            const bool stashed = c.cnt <= kStashCap;
            GenSums g;
            g.pre_w = g.pre_c = g.tot_w = g.tot_c = g.bad = 0;
            uint32_t ec = 0;
            bool direct_ok = false;
            if (!stashed) {
                // rare: more outliers than the stash holds.  Place the token now.
                uint32_t now[kEarly];
                request_generation<NW>(table + (it & 3u) * kFusedGridCap, gen_size(it), now);
                g = resolve_generation<NW>(table + (it & 3u) * kFusedGridCap, gen_size(it), wg, gen_tag(it),
                                           p.spin_limit, now, areas + (it & 1u) * kLdsResolve);
                failed |= g.bad;
                ec = base_c + g.pre_c;
                direct_ok = !g.bad && (uint64_t)ec + c.cnt <= p.outlier_capacity;
            }
            if (omask && (stashed || direct_ok)) {
                const uint16_t *raw = reinterpret_cast<const uint16_t *>(lrow + run * kRunLdsDw);
                uint32_t *stash = stashes + (it & 1u) * kStashCap;
                uint32_t pos = loff;
                uint32_t ev = omask & 0xFFFFu, od = omask >> 16;
                while (ev | od) {
                    const uint32_t je = ev ? 2u * (uint32_t)__builtin_ctz(ev) : 64u;
                    const uint32_t jo = od ? 2u * (uint32_t)__builtin_ctz(od) + 1u : 64u;
                    uint32_t j;
                    if (je < jo) { j = je; ev &= ev - 1u; } else { j = jo; od &= od - 1u; }
                    const uint32_t col = run * kRun + j;
                    if (stashed) {
                        stash[pos] = (col << 16) | raw[j];
                    } else {
                        out_col[(size_t)ec + pos] = (uint16_t)col;
                        out_val[(size_t)ec + pos] = raw[j];
                    }
                    ++pos;
                }
            }
            if (!stashed) {
                if (!g.bad) store_token(cur, g, false);
                base_w += g.tot_w;
                base_c += g.tot_c;
                placed = true;
            }
        }
        have_pending = !placed;
        pd = cur;

        if (tn < p.tokens) write_row();   // this wave is done with its part of the row
    }

    // ---- the last token of this workgroup
    GenSums g;
    g.pre_w = g.pre_c = g.tot_w = g.tot_c = g.bad = 0;
    if (have_pending) {
        uint32_t now[kEarly];
        if (NW > 1) __syncthreads();      // the stash of the last token is complete
#ifndef X_NORESOLVE
        request_generation<NW>(table + (pd.gen & 3u) * kFusedGridCap, gen_size(pd.gen), now);
        g = resolve_generation<NW>(table + (pd.gen & 3u) * kFusedGridCap, gen_size(pd.gen), wg, gen_tag(pd.gen),
                                   p.spin_limit, now, areas + (pd.gen & 1u) * kLdsResolve);
#endif
        failed |= g.bad;
        if (!g.bad) store_token(pd, g, true);
    }
    if (failed && tid == 0) {
        __hip_atomic_fetch_or(ctrl + kCtlError, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        write_header(p, blob, 0, 0, 6u);    // the header may already be final: overwrite it
    }
    // the workgroup that owns the last token closes the blob
    if (pd.token == p.tokens - 1u && tid == 0) {
        // totals: everything before the last generation plus the last generation itself; if the
        // last token was placed directly, base already contains its generation
        const uint64_t nnz = have_pending ? (uint64_t)base_c + g.tot_c : base_c;
        const uint64_t wordsum = have_pending ? (uint64_t)base_w + g.tot_w : base_w;
        row_ptr[p.tokens] = nnz;
        pay_off[p.tokens] = wordsum << 2;
        const uint32_t err = failed | __hip_atomic_load(ctrl + kCtlError, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        write_header(p, blob, nnz, wordsum << 2, err ? 6u : (nnz > p.outlier_capacity ? 3u : 0u));
        __hip_atomic_store(ctrl + kCtlError, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(ctrl + kCtlBank, bank ^ 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------- launchers

static hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

typedef void (*FusedKernel)(const Params, const uint16_t *, uint8_t *, uint8_t *);

template <int DT>
static FusedKernel fused_kernel_for(uint32_t nw) {
    switch (nw) {
        case 1: return k_fused<DT, 1>;
        case 2: return k_fused<DT, 2>;
        case 3: return k_fused<DT, 3>;
        case 4: return k_fused<DT, 4>;
        case 8: return k_fused<DT, 8>;
        default: return k_fused<DT, 16>;
    }
}

static FusedKernel fused_kernel(uint32_t dtype, uint32_t nw) {
    return dtype == (uint32_t)kF16 ? fused_kernel_for<kF16>(nw) : fused_kernel_for<kBF16>(nw);
}

// waves per workgroup of the fused kernel for a row of `runs` runs: the smallest instantiated size
uint32_t compress_waves(uint32_t runs) {
    const uint32_t need = (runs + 63u) / 64u;
    if (need <= 4) return need;
    return need <= 8 ? 8u : 16u;
}

int prepare_fused_kernels() {
    const int big = (int)(((kMaxHidden / kRun) * kRunLdsDw + kFusedScratchDw) * 4);
    static const uint32_t sizes[] = {1, 2, 3, 4, 8, 16};
    for (uint32_t dt = 0; dt < 2; ++dt)
        for (uint32_t nw : sizes) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fused_kernel(dt, nw)),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, big);
            if (e != hipSuccess) return (int)e;
        }
    return 0;
}

// Largest grid whose workgroups are all resident at once on the current device, for this plan.
int fused_resident_workgroups(const Params &p, const Geometry &g, uint32_t *out) {
    int dev = 0, cus = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(fused_kernel(p.dtype, g.waves)),
                                                         (int)(64u * g.waves), g.lds_fused_bytes);
    if (e != hipSuccess) return (int)e;
    if (per_cu < 1 || cus < 1) return (int)hipErrorInvalidConfiguration;
    *out = (uint32_t)per_cu * (uint32_t)cus;
    return 0;
}

int launch_fused(const Params &p, const Geometry &g, uint32_t grid, const void *d_in, void *d_blob, void *d_ws,
                 void *stream) {
    hipLaunchKernelGGL(fused_kernel(p.dtype, g.waves), dim3(grid), dim3(64u * g.waves), g.lds_fused_bytes,
                       as_stream(stream), p, static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                       static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------- workspace reset

__global__ void k_ws_reset(const Params p, uint8_t *__restrict__ ws) {
    uint32_t *table = reinterpret_cast<uint32_t *>(ws + p.ws_agg);
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 2u * 4u * kFusedGridCap) table[i] = 0;
    if (i < 64) ctrl[i] = 0;
}

int launch_ws_reset(const Params &p, void *d_ws, void *stream) {
    const uint32_t n = 2u * 4u * kFusedGridCap;
    hipLaunchKernelGGL(k_ws_reset, dim3((n + 255) / 256), dim3(256), 0, as_stream(stream), p,
                       static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

}  // namespace tsq
