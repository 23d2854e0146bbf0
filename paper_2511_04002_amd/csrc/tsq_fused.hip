// Single-pass compress kernel (gfx950): Eq. (ts), Algorithm 1, Eq. (Proposed), bit packing and
// CSR emission with ONE read of the input.
//
// A persistent grid of G workgroups.  Workgroup g starts with token g; every further token comes
// from a ticket counter.  The workgroups are spread over C classes (g % C), class c owns the
// tokens t with t % C == c and hands them out in ascending order from its own counter, so that
// no counter sees more than one atomic per C tokens (atomics on one address are slow across the
// chip's eight dies) and a workgroup that is slowed down simply takes fewer tokens.
//
// Placement of the variable-length outputs (payload words, CSR entries) needs the exclusive
// prefix over all earlier tokens.  A workgroup publishes, per token, one 32-bit word (words,
// outliers) in a per-token table.  A workgroup's tokens ascend, so it keeps the sum over the
// tokens it has already seen and, for each new token of its own, one of its waves reads the
// table words of the tokens in between (about G of them).  Nobody scans on behalf of the others,
// nothing forms a serial chain, and apart from the tickets there are no atomic read-modify-write
// operations (on this chip they cost microseconds when several dies touch one address).
//
// To keep the wait for slower neighbours off the critical path a token is stored almost two
// iterations late: iteration i computes token i, publishes it, stores token i-2, and only then
// packs token i's codes into the payload
// image in LDS that token i-2 occupied (two images and two outlier stashes alternate).  All
// earlier tokens were handed out before token i-2 was, so by then they have been published.  The row of iteration i+1 is fetched into
// registers in the middle of iteration i; its ticket was requested an iteration earlier.
//
// Progress: the smallest token that is not stored yet has all its predecessors published, and if
// nobody has taken it yet, no workgroup of its class is waiting (their pending tokens would be
// smaller); so some workgroup can always move.  Every wait is bounded by p.spin_limit anyway; an
// expired wait marks the blob as failed (TSQ_ERR_INTERNAL) instead of hanging.
//
// Per-call state: table words carry a 2-bit tag of the call (epoch % 3 + 1), so a word of an
// earlier call is never taken for a current one; the ticket counters exist in two banks
// (epoch & 1).  The workgroup that stores the last token waits until every workgroup has
// drawn its final (failing) ticket, clears the other bank for the next call and advances the epoch.
#include <hip/hip_runtime.h>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

enum { kCtlEpoch = 0, kCtlError = 1 };
constexpr uint32_t kNoToken = 0xFFFFFFFFu;

// Table word: bits 31..30 = tag of the call (0 = never written), bits 29..16 = payload words of
// the token (<= 8192), bits 15..0 = its outliers (<= 32768).
__device__ __forceinline__ uint32_t word_load(const uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void word_store(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One more round of a bounded wait: false when the limit is reached or another workgroup has
// already given up (checked now and then, so that a broken run ends quickly everywhere).
__device__ __forceinline__ bool keep_waiting(uint32_t &spins, uint32_t limit, const uint32_t *error_flag) {
    if (++spins >= limit) return false;
    if ((spins & 255u) == 0 && __hip_atomic_load(error_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return false;
    __builtin_amdgcn_s_sleep(2);
    return true;
}

struct __attribute__((packed, aligned(4))) Dw4 { uint32_t a, b, c, d; };   // 16 bytes at a 4-byte aligned address

// ---- the row in LDS, fused kernel: 16 dwords per run, no padding.  The four 16-byte chunks of
// run r are stored in the order k ^ ((r >> 1) & 3), which spreads eight neighbouring runs over
// all 32 banks for 16-byte accesses. ----
template <bool FULL>
__device__ __forceinline__ void write_row_part_sw(uint32_t *lrow, uint32_t runs, const RowPart &pre) {
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
    const uint32_t q0 = 256u * wv + lane;                  // first 16-byte piece of the row this lane moves
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t q = q0 + 64u * k, r = q >> 2, c = (q & 3u) ^ ((r >> 1) & 3u);
        if (FULL || r < runs)
            *reinterpret_cast<uint4 *>(lrow + r * 16u + c * 4u) =
                make_uint4(pre.w[4 * k], pre.w[4 * k + 1], pre.w[4 * k + 2], pre.w[4 * k + 3]);
    }
}
__device__ __forceinline__ void load_run_sw(const uint32_t *lrow, uint32_t r, uint32_t (&w)[16]) {
    const uint32_t sw = (r >> 1) & 3u;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        const uint4 q = *reinterpret_cast<const uint4 *>(lrow + r * 16u + ((k ^ sw) << 2));
        w[4 * k] = q.x; w[4 * k + 1] = q.y; w[4 * k + 2] = q.z; w[4 * k + 3] = q.w;
    }
}
__device__ __forceinline__ uint32_t raw_element_sw(const uint32_t *lrow, uint32_t r, uint32_t j) {
    // byte 2j of the run, its 16-byte chunk index xor-ed with the run's swizzle: the run's part of
    // the address does not depend on j
    const uint32_t at = ((r * 64u) | (((r >> 1) & 3u) << 4)) ^ (j << 1);
    return *reinterpret_cast<const uint16_t *>(reinterpret_cast<const uint8_t *>(lrow) + at);
}

// nd dwords of packed codes of a run into the token's payload image in LDS
template <int B, bool FULL>
__device__ __forceinline__ void put_codes(uint32_t *dst, const uint32_t (&o)[8], uint32_t nd) {
    if (FULL || nd >= (uint32_t)B) {
        int k = 0;
        // the image is 16-byte aligned and run*B dwords in: use the widest stores the alignment allows
        if (B % 4 == 0) {
#pragma unroll
            for (; k + 4 <= B; k += 4) *reinterpret_cast<uint4 *>(dst + k) = make_uint4(o[k], o[k + 1], o[k + 2], o[k + 3]);
        } else if (B % 2 == 0) {
#pragma unroll
            for (; k + 2 <= B; k += 2) *reinterpret_cast<uint2 *>(dst + k) = make_uint2(o[k], o[k + 1]);
        } else {
#pragma unroll
            for (; k < B; ++k) dst[k] = o[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < B; ++k)
            if ((uint32_t)k < nd) dst[k] = o[k];
    }
}
template <int B, bool FULL>
__device__ __forceinline__ void pack_to_image(const uint32_t (&m)[8], const uint32_t (&w)[16], uint32_t *dst,
                                              uint32_t nd) {
    uint32_t o[8];
    {
        uint32_t t[B];
        pack_regs<B>(m, w, t);
#pragma unroll
        for (int k = 0; k < B; ++k) o[k] = t[k];
    }
    put_codes<B, FULL>(dst, o, nd);
}

// ---- placement ----
// What a workgroup knows about the tokens before one of its own.
struct Place {
    uint32_t done;           // tokens 0 .. done-1 are contained in base_*
    uint32_t base_w, base_c; // their payload words / outliers
};
struct Prefix {
    uint32_t ew, ec;         // payload words / outliers of all tokens before the token
    uint32_t bad;            // a wait expired
};

// Exclusive prefix of token t (t >= pl.done), in two steps so that the memory latency of the
// table reads overlaps with other work: place_request asks for the table words of the tokens
// pl.done .. t-1 (kEarly per thread; all waves take part), place_finish waits for those that
// were not published yet, reads what lies beyond kEarly words per thread, and adds up.
// area: 3*kMaxWaves dwords.  All threads of the block call both (one barrier, NW > 1).
constexpr int kEarly = 4;
__device__ __forceinline__ uint32_t dot_halves(uint32_t v, uint32_t sel, uint32_t acc) {
    // v.lo * sel.lo + v.hi * sel.hi + acc in one instruction
    return __builtin_amdgcn_udot2(__builtin_bit_cast(u16x2, v), __builtin_bit_cast(u16x2, sel), acc, false);
}
template <int NW>
__device__ __forceinline__ void place_request(const uint32_t *sizes, uint32_t tag, uint32_t t, const Place &pl,
                                              uint32_t (&v)[kEarly]) {
#pragma unroll
    for (int k = 0; k < kEarly; ++k) {
        const uint32_t j = pl.done + (uint32_t)k * 64u * NW + threadIdx.x;
        v[k] = tag << 30;                 // "published, empty" for positions past the range
        if (j < t) v[k] = word_load(sizes + j);
    }
}
template <int NW>
__device__ __forceinline__ Prefix place_finish(const Params &p, const uint32_t *sizes, uint32_t tag, uint32_t t,
                                               Place &pl, const uint32_t (&v)[kEarly], uint32_t *area,
                                               uint32_t *error_flag) {
    constexpr uint32_t kThreads = 64u * NW;
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
    const uint32_t tag3 = tag << 30;
    uint32_t w[kEarly];
    uint32_t differ = 0, bad = 0;
#pragma unroll
    for (int k = 0; k < kEarly; ++k) { w[k] = v[k]; differ |= w[k] ^ tag3; }
    if (differ >> 30) {
        // some word does not carry this call's tag yet: wait for it
#pragma unroll
        for (int k = 0; k < kEarly; ++k) {
            const uint32_t j = pl.done + (uint32_t)k * kThreads + threadIdx.x;
            uint32_t spins = 0;
            while ((w[k] >> 30) != tag && keep_waiting(spins, p.spin_limit, error_flag)) w[k] = word_load(sizes + j);
            if ((w[k] >> 30) != tag) { bad = 1; w[k] = tag3; }
        }
    }
    // sums of the low halves (outliers) and of the high halves (tag | words): one dot product each
    uint32_t sc = 0, sh = 0;
#pragma unroll
    for (int k = 0; k < kEarly; ++k) {
        sc = dot_halves(w[k], 0x00000001u, sc);
        sh = dot_halves(w[k], 0x00010000u, sh);
    }
    uint32_t sw = sh - (uint32_t)kEarly * (tag << 14);       // the tags that rode along in the high halves
    // what lies beyond the early words (narrow workgroups, whose grid is large): four loads in flight
    for (uint32_t j0 = pl.done + kEarly * kThreads + threadIdx.x; j0 < t; j0 += 4u * kThreads) {
        uint32_t x[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t j = j0 + (uint32_t)k * kThreads;
            x[k] = tag3;
            if (j < t) x[k] = word_load(sizes + j);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t j = j0 + (uint32_t)k * kThreads;
            uint32_t spins = 0;
            while ((x[k] >> 30) != tag && keep_waiting(spins, p.spin_limit, error_flag)) x[k] = word_load(sizes + j);
            if ((x[k] >> 30) != tag) { bad = 1; x[k] = 0; }
            sw += (x[k] >> 16) & 0x3FFFu;
            sc += x[k] & 0xFFFFu;
        }
    }

    uint32_t r0 = wave_sum_u32(sw), r1 = wave_sum_u32(sc);
    uint32_t r2 = __builtin_amdgcn_ballot_w64(bad != 0) != 0 ? 1u : 0u;
    if (r2 && lane == 0) __hip_atomic_fetch_or(error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (NW > 1) {
        if (lane == 0) { area[wv] = r0; area[kMaxWaves + wv] = r1; area[2 * kMaxWaves + wv] = r2; }
        __syncthreads();
        uint32_t a0 = 0, a1 = 0, a2 = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) { a0 += area[w]; a1 += area[kMaxWaves + w]; a2 |= area[2 * kMaxWaves + w]; }
        r0 = uniform(a0); r1 = uniform(a1); r2 = uniform(a2);
    }
    pl.done = t;
    pl.base_w += r0;
    pl.base_c += r1;
    Prefix x;
    x.ew = pl.base_w;
    x.ec = pl.base_c;
    x.bad = r2;
    return x;
}

// One ticket of a class counter; the caller needs the result an iteration later.  The address goes
// through a register the compiler knows nothing about (the offset is zero): an address that is
// the same in every lane would have the atomic rewritten into a wave-wide reduction whose result
// is read, and so waited for, on the spot.
__device__ __forceinline__ uint32_t draw_ticket(uint32_t *counter) {
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    return __hip_atomic_fetch_add(counter + zero, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What a workgroup keeps of a token between computing it and storing it.
struct Pending {
    uint32_t width, cnt, words, token;
    uint32_t parity;   // which payload image and which stash hold it
};

// Where a token's outputs go, and the LDS areas they come from.
struct StoreTargets {
    uint64_t *pay_off, *row_ptr;
    uint32_t *payload;
    uint16_t *out_col, *out_val;
    const uint32_t *images, *stashes;
    uint32_t runs;
    uint64_t payload_words, outlier_capacity;
};
// What the workgroup that stores the very last token needs to close the blob.
struct Tail {
    uint32_t token, ew, ec, words, cnt;
};

// Stores a token whose prefix is known: the payload image LDS -> HBM (16 bytes per thread and
// step, contiguous over the workgroup), its offsets, and (from_stash) its outliers.  The image
// and the stash were written by all waves: a barrier lies between their writes and this call.
// Returns false without storing anything if the payload would leave its section, whatever the
// table said.
template <int NW>
__device__ __forceinline__ bool store_token(const StoreTargets &o, const Pending &q, const Prefix &x, bool from_stash,
                                            Tail &tail) {
    constexpr uint32_t kThreads = 64u * NW;
    // the thread index through a register the compiler knows nothing about: the addresses derived
    // from it are computed here, not once before the token loop and then kept (or spilled) across it
    uint32_t tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    if ((uint64_t)x.ew + q.words > o.payload_words) return false;
    if (tid == 0) {
        o.pay_off[q.token] = (uint64_t)x.ew << 2;
        o.row_ptr[q.token] = x.ec;
    }
    // Every address below is a uniform base (x is uniform) plus a byte offset of 32 bits: the base
    // stays in scalar registers and no thread holds a 64-bit pointer of its own.
    const uint32_t *img = o.images + q.parity * o.runs * 8u;
    uint8_t *dst = reinterpret_cast<uint8_t *>(o.payload + x.ew);
    const uint32_t quads = q.words >> 2;      // at most 2 * kThreads: 8 bits x 32 elements per thread = 32 bytes
    const __amdgpu_buffer_rsrc_t window = raw_window(dst, q.words << 2);
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) {
        const uint32_t i = tid + r * kThreads;
        if (i < quads) {
            // written through the L2 as it goes (the payload is what decompress reads next: it should stay
            // in the memory-side cache, which a streaming store would bypass; a plain store would leave
            // it dirty in the L2 until the end of the kernel, where writing it back costs about 2 us)
            const u32x4 v = *reinterpret_cast<const u32x4 *>(img + 4u * i);
            store_quad_through(window, 16u * i, v);
        }
    }
    const uint32_t rest = q.words & 3u;
    if (tid < rest) *reinterpret_cast<uint32_t *>(dst + 4u * (4u * quads + tid)) = img[4u * quads + tid];
    if (from_stash && q.cnt > 0 && (uint64_t)x.ec + q.cnt <= o.outlier_capacity) {
        const uint32_t *stash = o.stashes + q.parity * kStashCap;
        uint8_t *col = reinterpret_cast<uint8_t *>(o.out_col + x.ec), *val = reinterpret_cast<uint8_t *>(o.out_val + x.ec);
        for (uint32_t k = tid; k < q.cnt; k += kThreads) {
            const uint32_t e = stash[k];
            *reinterpret_cast<uint16_t *>(col + 2u * k) = (uint16_t)(e >> 16);
            *reinterpret_cast<uint16_t *>(val + 2u * k) = (uint16_t)e;
        }
    }
    tail.token = q.token; tail.ew = x.ew; tail.ec = x.ec; tail.words = q.words; tail.cnt = q.cnt;
    return true;
}

// LDS map (dynamic): row: runs*16 | two payload images: runs*8 each | ring: 4 reduce areas |
// 4 placement areas (used in rotation, like the reduce areas) | 2 ticket slots (8 dwords) | two stashes
constexpr uint32_t kLdsRing = 4 * 2 * kMaxWaves, kLdsPlace = 3 * kMaxWaves;
static_assert(kFusedScratchDw == kLdsRing + 4 * kLdsPlace + 8 + 2 * kStashCap, "LDS map of the fused kernel");

// FULL: the row fills the workgroup exactly (hidden == 2048 * NW), so every lane owns a whole run
// and none of the range checks of the general case is needed.
template <int DT, int NW, bool FULL>
__global__ void __launch_bounds__(64 * NW, 4)
k_fused(const Params p, const uint16_t *__restrict__ in, uint8_t *__restrict__ blob, uint8_t *__restrict__ ws) {
    extern __shared__ __align__(16) uint32_t lds[];
    constexpr uint32_t kThreads = 64 * NW;
    uint32_t *lrow = lds;
    const uint32_t runs = FULL ? 64u * NW : p.runs, pieces = FULL ? 256u * NW : p.pieces;
    uint32_t *images = lds + runs * 16u;                    // packed codes of the current and the pending token
    uint32_t *ring = images + 2u * runs * 8u;
    uint32_t *areas = ring + kLdsRing;
    uint32_t *tslot = areas + 4 * kLdsPlace;                // next token, one slot per iteration parity
    uint32_t *stashes = tslot + 8;                          // 2 x kStashCap dwords: col << 16 | raw value
    const uint32_t tid = threadIdx.x, run = tid;
    const uint32_t wg = blockIdx.x, G = gridDim.x;
    const bool owns = FULL || run < runs;
    const uint32_t left = FULL ? 4u : (owns ? pieces - 4 * run : 0);   // 16-byte pieces of the lane's run inside the row

    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint32_t epoch = uniform(ctrl[kCtlEpoch]);
    const uint32_t bank = epoch & 1u, tag = epoch % 3u + 1u;
    uint32_t *sizes = reinterpret_cast<uint32_t *>(ws + p.ws_sizes);
    uint32_t *tickets = reinterpret_cast<uint32_t *>(ws + p.ws_tickets) + (size_t)bank * kTicketClasses * kTicketStride;

    // ticket class of this workgroup: class c owns the tokens t % C == c; its first Wc tokens go to
    // its Wc workgroups without a ticket (workgroup g starts with token g)
    const uint32_t C = p.fused_classes, cls = wg % C;
    const uint32_t n_cls = (p.tokens - cls + C - 1u) / C;   // tokens of the class
    const uint32_t w_cls = (G - cls + C - 1u) / C;          // workgroups of the class
    uint32_t *counter = tickets + cls * kTicketStride;

    uint8_t *bits = blob + p.off_bits;
    float *scale = reinterpret_cast<float *>(blob + p.off_scale);
    uint64_t *pay_off = reinterpret_cast<uint64_t *>(blob + p.off_pay_off);
    uint64_t *row_ptr = reinterpret_cast<uint64_t *>(blob + p.off_row_ptr);
    uint32_t *payload = reinterpret_cast<uint32_t *>(blob + p.off_payload);
    uint16_t *out_col = reinterpret_cast<uint16_t *>(blob + p.off_out_col);
    uint16_t *out_val = reinterpret_cast<uint16_t *>(blob + p.off_out_val);

    // the row of the next iteration on its way HBM -> registers -> LDS (each wave its own part)
    RowPart pre;
    const uint32_t hidden = FULL ? 2048u * NW : p.hidden;

    Place pl;
    pl.done = 0; pl.base_w = 0; pl.base_c = 0;
    uint32_t failed = 0, turn = 0, pturn = 0;   // turn / pturn: rotation through the reduce / placement areas
    // tokens computed but not stored yet: `young` is from the previous iteration, `old` from the one
    // before.  A token's payload image and stash are those of its iteration's parity, so `old` has
    // to leave before the current token's codes are packed into the same image.
    Pending young, old;
    bool have_young = false, have_old = false;
    young.width = 8; young.cnt = 0; young.words = 0; young.token = 0; young.parity = 0;
    old = young;
    Tail tail;
    tail.token = kNoToken; tail.ew = tail.ec = tail.words = tail.cnt = 0;

    const StoreTargets out{pay_off, row_ptr, payload, out_col, out_val, images, stashes, runs,
                           p.payload_capacity >> 2, p.outlier_capacity};

    // ---- first token: the workgroup's own id; its row; the ticket of the second token
    uint32_t t = wg;                       // the grid never exceeds the token count
    fetch_row_part<FULL>(reinterpret_cast<const uint4 *>(row_address(p, in, t, hidden)), pieces, pre);
    uint32_t req = 0;                      // thread 0: the ticket in flight
    bool requesting = true;                // uniform: a ticket is in flight
    if (tid == 0) req = draw_ticket(counter);
    write_row_part_sw<FULL>(lrow, runs, pre);

    uint32_t it = 0;
    for (; t != kNoToken; ++it) {
        // ---- the ticket requested an iteration ago: the token after this one; ask for the one after that
        if (tid == 0) {
            uint32_t tn = kNoToken;
            if (requesting) {
                const uint32_t k = w_cls + req;
                if (k < n_cls) {
                    tn = k * C + cls;
                    req = draw_ticket(counter);
                }
            }
            tslot[it & 1u] = tn;
        }

        // the table words before the older pending token: asked for now, used after the width search
        uint32_t early[kEarly];
        if (have_old) place_request<NW>(sizes, tag, old.token, pl, early);

        // ---- Eq. (ts) and Algorithm 1 for token t
        Mags<DT> mg;
        uint32_t omask = 0, amax_bits = 0;
        {
            uint32_t w[16];
            load_run_sw(lrow, owns ? run : 0u, w);
            split_regs<DT, true>(w, p.thr_pk, mg, omask, amax_bits);
        }
        if (!owns) omask = 0;
        uint32_t m[8], cnt_before;
        // The width search is where the waves of a workgroup meet at barriers (one per cross-wave
        // reduction).  A compute unit's SIMDs each hold one wave of several workgroups; with the waves
        // of the workgroup that is in this phase preferred by the instruction arbiter, they reach
        // each barrier together instead of each being held up by whatever its SIMD's other waves
        // happen to do, and less time is lost waiting there (5 % of the kernel on 8192 x 8192).
        __builtin_amdgcn_s_setprio(1);
        const Choice c = choose_width<DT, NW>(p, mg, omask, amax_bits, owns, ring, turn, m, cnt_before);
        __builtin_amdgcn_s_setprio(0);
        const uint32_t tn = uniform(tslot[it & 1u]);     // written before the barrier inside choose_width
        requesting = tn != kNoToken;
        const uint32_t words = row_bytes(p.hidden, c.width) >> 2;
        if (tid == 0) {
            word_store(sizes + t, (tag << 30) | (words << 16) | c.cnt);
            bits[t] = (uint8_t)c.width;
            scale[t] = scale_of(c.amax, c.width);
        }
        // the next row starts its way from HBM now that the registers of the width search are free
        if (tn != kNoToken)
            fetch_row_part<FULL>(reinterpret_cast<const uint4 *>(row_address(p, in, tn, hidden)), pieces, pre);

        // ---- store the token of two iterations ago: its image and stash are needed now
        if (have_old) {
            const Prefix x = place_finish<NW>(p, sizes, tag, old.token, pl, early, areas + (pturn++ & 3u) * kLdsPlace,
                                              ctrl + kCtlError);
            failed |= x.bad;
            if (!x.bad && !store_token<NW>(out, old, x, true, tail)) failed = 1;
            have_old = false;
            if (NW > 1) __syncthreads();      // the image and the stash of this parity are free again
        }

        // ---- codes of the lane's run at the chosen width, into this iteration's payload image
        Pending cur;
        cur.width = c.width; cur.cnt = c.cnt; cur.words = words; cur.token = t; cur.parity = it & 1u;
        if (owns) {
            uint32_t wr[16];
            load_run_sw(lrow, run, wr);
            uint32_t *dst = images + cur.parity * runs * 8u + run * c.width;
            const uint32_t nd = (FULL || left >= 4) ? c.width : ((left * c.width + 3u) >> 2);
            switch (c.width) {
                case 2: pack_to_image<2, FULL>(m, wr, dst, nd); break;
                case 3: pack_to_image<3, FULL>(m, wr, dst, nd); break;
                case 4: pack_to_image<4, FULL>(m, wr, dst, nd); break;
                case 5: pack_to_image<5, FULL>(m, wr, dst, nd); break;
                case 6: pack_to_image<6, FULL>(m, wr, dst, nd); break;
                case 7: pack_to_image<7, FULL>(m, wr, dst, nd); break;
                default: pack_to_image<8, FULL>(m, wr, dst, nd); break;
            }
        }

        // ---- T_above of token t: into this iteration's stash in column order, or straight out if
        //      it is too long for the stash
        bool placed = false;
        if (c.cnt > 0) {
            const uint32_t nl = (uint32_t)__builtin_popcount(omask);
            const uint32_t loff = cnt_before + wave_incl_scan_u32(nl) - nl;
            const bool stashed = c.cnt <= kStashCap;
            Prefix x;
            x.ew = x.ec = x.bad = 0;
            bool direct_ok = false;
            if (!stashed) {
                // rare: more outliers than the stash holds.  Place everything that is pending, then
                // this token, now.
                uint32_t now[kEarly];
                if (have_young) {
                    place_request<NW>(sizes, tag, young.token, pl, now);
                    const Prefix y = place_finish<NW>(p, sizes, tag, young.token, pl, now,
                                                      areas + (pturn++ & 3u) * kLdsPlace, ctrl + kCtlError);
                    failed |= y.bad;
                    if (!y.bad && !store_token<NW>(out, young, y, true, tail)) failed = 1;
                    have_young = false;
                }
                place_request<NW>(sizes, tag, t, pl, now);
                x = place_finish<NW>(p, sizes, tag, t, pl, now, areas + (pturn++ & 3u) * kLdsPlace, ctrl + kCtlError);
                failed |= x.bad;
                direct_ok = !x.bad && (uint64_t)x.ec + c.cnt <= p.outlier_capacity;
            }
            if (omask && (stashed || direct_ok)) {
                uint32_t *stash = stashes + (it & 1u) * kStashCap;
                uint32_t pos = loff;
                for (uint32_t rest = omask; rest; rest &= rest - 1u) {
                    const uint32_t j = (uint32_t)__builtin_ctz(rest);
                    const uint32_t col = run * kRun + j;
                    if (stashed) {
                        stash[pos] = (col << 16) | raw_element_sw(lrow, run, j);
                    } else {
                        out_col[(size_t)x.ec + pos] = (uint16_t)col;
                        out_val[(size_t)x.ec + pos] = (uint16_t)raw_element_sw(lrow, run, j);
                    }
                    ++pos;
                }
            }
            if (!stashed) {
                if (!x.bad && !store_token<NW>(out, cur, x, false, tail)) failed = 1;
                placed = true;
            }
        }
        old = young; have_old = have_young;
        young = cur; have_young = !placed;

        if (tn != kNoToken) write_row_part_sw<FULL>(lrow, runs, pre);   // this wave is done with its part of the row
        t = tn;
    }

    // ---- the tokens still pending, oldest first
    if (have_old) {
        uint32_t now[kEarly];
        place_request<NW>(sizes, tag, old.token, pl, now);
        const Prefix x = place_finish<NW>(p, sizes, tag, old.token, pl, now, areas + (pturn++ & 3u) * kLdsPlace,
                                          ctrl + kCtlError);
        failed |= x.bad;
        if (!x.bad && !store_token<NW>(out, old, x, true, tail)) failed = 1;
    }
    if (have_young) {
        uint32_t now[kEarly];
        place_request<NW>(sizes, tag, young.token, pl, now);
        const Prefix x = place_finish<NW>(p, sizes, tag, young.token, pl, now, areas + (pturn++ & 3u) * kLdsPlace,
                                          ctrl + kCtlError);
        failed |= x.bad;
        if (!x.bad && !store_token<NW>(out, young, x, true, tail)) failed = 1;
    }
    if (failed && tid == 0) write_header(p, blob, 0, 0, 6u);   // the header may already be final: overwrite it

    // ---- the workgroup that stored the last token closes the blob and prepares the next call
    if (tail.token == p.tokens - 1u) {
        const uint64_t nnz = (uint64_t)tail.ec + tail.cnt, wordsum = (uint64_t)tail.ew + tail.words;
        // every workgroup draws exactly one failing ticket, after which all counters add up to the
        // token count; until then somebody may not even have read the epoch yet
        uint32_t spins = 0, drawn = 0;
        for (;;) {
            uint32_t v = 0;
            if ((tid & 63u) < C) v = word_load(tickets + (tid & 63u) * kTicketStride);
            drawn = wave_sum_u32(v);                          // C <= 64 classes: one lane each
            if (drawn == p.tokens || !keep_waiting(spins, p.spin_limit, ctrl + kCtlError)) break;
        }
        const bool late = drawn != p.tokens;
        uint32_t *tickets_next =
            reinterpret_cast<uint32_t *>(ws + p.ws_tickets) + (size_t)(1u - bank) * kTicketClasses * kTicketStride;
        for (uint32_t i = tid; i < kTicketClasses; i += kThreads) tickets_next[i * kTicketStride] = 0;
        if (tid == 0) {
            row_ptr[p.tokens] = nnz;
            pay_off[p.tokens] = wordsum << 2;
            const uint32_t err = failed | (late ? 1u : 0u) |
                                 __hip_atomic_load(ctrl + kCtlError, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            write_header(p, blob, nnz, wordsum << 2, err ? 6u : (nnz > p.outlier_capacity ? 3u : 0u));
            __hip_atomic_store(ctrl + kCtlError, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(ctrl + kCtlEpoch, epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ---------------------------------------------------------------- launchers

static hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

typedef void (*FusedKernel)(const Params, const uint16_t *, uint8_t *, uint8_t *);

template <int DT, bool FULL>
static FusedKernel fused_kernel_for(uint32_t nw) {
    switch (nw) {
        case 1: return k_fused<DT, 1, FULL>;
        case 2: return k_fused<DT, 2, FULL>;
        case 3: return k_fused<DT, 3, FULL>;
        case 4: return k_fused<DT, 4, FULL>;
        case 8: return k_fused<DT, 8, FULL>;
        default: return k_fused<DT, 16, FULL>;
    }
}

static FusedKernel fused_kernel(uint32_t dtype, uint32_t nw, bool full) {
    if (full) return dtype == (uint32_t)kF16 ? fused_kernel_for<kF16, true>(nw) : fused_kernel_for<kBF16, true>(nw);
    return dtype == (uint32_t)kF16 ? fused_kernel_for<kF16, false>(nw) : fused_kernel_for<kBF16, false>(nw);
}
static bool fills_workgroup(const Params &p, const Geometry &g) { return p.hidden == 2048u * g.waves; }

// waves per workgroup of the fused kernel for a row of `runs` runs: the smallest instantiated size
uint32_t compress_waves(uint32_t runs) {
    const uint32_t need = (runs + 63u) / 64u;
    if (need <= 4) return need;
    return need <= 8 ? 8u : 16u;
}

int prepare_fused_kernels() {
    const int big = (int)(((kMaxHidden / kRun) * 32u + kFusedScratchDw) * 4);
    static const uint32_t sizes[] = {1, 2, 3, 4, 8, 16};
    for (uint32_t dt = 0; dt < 2; ++dt)
        for (uint32_t nw : sizes)
            for (int full = 0; full < 2; ++full) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fused_kernel(dt, nw, full != 0)),
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
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(fused_kernel(p.dtype, g.waves, fills_workgroup(p, g))),
                                                         (int)(64u * g.waves), g.lds_fused_bytes);
    if (e != hipSuccess) return (int)e;
    if (per_cu < 1 || cus < 1) return (int)hipErrorInvalidConfiguration;
    *out = (uint32_t)per_cu * (uint32_t)cus;
    return 0;
}

int launch_fused(const Params &p, const Geometry &g, uint32_t grid, const void *d_in, void *d_blob, void *d_ws,
                 void *stream) {
    hipLaunchKernelGGL(fused_kernel(p.dtype, g.waves, fills_workgroup(p, g)), dim3(grid), dim3(64u * g.waves), g.lds_fused_bytes,
                       as_stream(stream), p, static_cast<const uint16_t *>(d_in), static_cast<uint8_t *>(d_blob),
                       static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------- workspace reset

__global__ void k_ws_reset(const Params p, uint8_t *__restrict__ ws) {
    uint32_t *sizes = reinterpret_cast<uint32_t *>(ws + p.ws_sizes);
    uint32_t *tickets = reinterpret_cast<uint32_t *>(ws + p.ws_tickets);
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < p.tokens; i += stride) sizes[i] = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < 2u * kTicketClasses * kTicketStride; i += stride)
        tickets[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x < 64) ctrl[threadIdx.x] = 0;
}

int launch_ws_reset(const Params &p, void *d_ws, void *stream) {
    uint32_t blocks = (p.tokens + 255u) / 256u;
    if (blocks < 32) blocks = 32;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_ws_reset, dim3(blocks), dim3(256), 0, as_stream(stream), p, static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

}  // namespace tsq
