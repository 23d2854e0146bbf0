// Single-pass compress kernel (gfx950): Eq. (ts), Algorithm 1, Eq. (Proposed), bit packing and
// CSR emission with ONE read of the input.
//
// Workgroup 0 is the scanner: up to four of its waves turn the per-token sizes, as they are
// published, into the device-wide exclusive prefix (the exclusive scan that places the
// variable-length outputs).  Every other workgroup computes tokens.  All tokens are handed
// out by ticket counters, so a workgroup that has not started yet holds nothing that anybody
// waits for (workgroups are dispatched in index order, so workgroup 0 is the first to start).
//
// Tickets: the computing workgroups are spread over C classes (g % C), class c owns the
// tokens t with t % C == c and hands them out in ascending order from its own counter, so no
// counter sees more than one atomic per C tokens (atomics on one address are slow across the
// chip's eight dies) and a workgroup that is slowed down simply takes fewer tokens.  The
// counter's top byte carries the call's epoch (mod 3), so the first ticket also tells the
// workgroup which tag the tables of this call use.
//
// Per token a workgroup publishes one 32-bit word (tag, payload words, outliers) in a table.
// The scanner reads the table in order, 512 or 1024 words per round, and for the leading run of
// published tokens writes (tag, words before, outliers before) into a second table, and the
// blob's pay_off / row_ptr entries on the way.  Nobody else adds anything up.  (One wave alone
// does not keep up with 200 tokens per microsecond: its rounds are chains of dependent steps.)
//
// A token is stored two iterations after it was computed: iteration i computes token i,
// publishes it, stores token i-2 and then packs token i's codes into the payload image in LDS
// that token i-2 occupied (two images and two outlier stashes alternate).  By then every
// earlier token was handed out at least two iterations ago, so its prefix is there.  Each
// wave stores the part of the image and of the stash that it wrote itself: nothing between the
// width search of one token and that of the next needs a workgroup barrier.  A wave with more
// outliers than its stash holds (rare) keeps none of them and takes them from the row again
// when the token is stored.
//
// Progress: a workgroup's tokens ascend, and what it waits for is the prefix of a token older
// than the one it is computing.  So the smallest unpublished token is either being computed
// (if its workgroup waits, then for a prefix that depends on published tokens only, and the
// scanner waits for publications only), or not yet drawn, and then the workgroups of its class
// hold older tokens only and one of them draws it.  That holds for one such kernel on the
// device, with at least one workgroup of every class running; two of these kernels at once, each
// with workgroups that have not started, can hold the slots that the other one's workgroups
// need (the host side orders such launches).  Every wait is bounded by p.spin_limit anyway; an
// expired wait raises the workspace's error word, which ends every other wait quickly, and the
// scanner then writes status TSQ_ERR_INTERNAL.  The scanner alone writes the header.
//
// End of a call: every wave adds one to its class's count of finished waves; the scanner waits
// for all of them, writes the totals and the header, and puts the counters into the state the
// next call expects (next epoch, no tickets drawn).
#include <hip/hip_runtime.h>

#include <mutex>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

constexpr uint32_t kNoToken = 0xFFFFFFFFu;
constexpr uint32_t kTicketBits = 24, kTicketMask = (1u << kTicketBits) - 1u;
enum { kCntTickets = 0, kCntDone = 1 };      // words of a class's counter line

// Table word: bits 31..30 = tag of the call (0 = never written), bits 29..26 = width of the token,
// bits 15..0 = its outliers (<= 32768).
// Prefix word: bits 63..62 = tag, bits 61..32 = payload words before the token, bits 31..0 =
// outliers before the token.
__device__ __forceinline__ uint32_t word_load(const uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void word_store(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t prefix_load(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void prefix_store(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// A zero the compiler knows nothing about, in a vector register: an address formed with it is
// not provably the same in every lane, so loads and atomics through it stay vector operations
// that go to memory (a provably uniform one may become a scalar load, or a wave-wide reduction
// whose result is waited for on the spot).
__device__ __forceinline__ uint32_t opaque_zero() {
    uint32_t zero = 0;
    asm volatile("" : "+v"(zero));
    return zero;
}

// A uniform value that the compiler is to keep as it is now, instead of deriving it again from its (wider)
// sources wherever it is used.
__device__ __forceinline__ uint32_t as_computed(uint32_t v) {
    asm volatile("" : "+s"(v));
    return v;
}

// One more round of a bounded wait: false when the limit is reached or somebody has already
// given up (checked now and then, so that a broken run ends quickly everywhere).
__device__ __forceinline__ bool keep_waiting(uint32_t &spins, uint32_t limit, const uint32_t *error_flag) {
    if (++spins >= limit) return false;
    if ((spins & 255u) == 0 && __hip_atomic_load(error_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return false;
    __builtin_amdgcn_s_sleep(2);
    return true;
}
__device__ __forceinline__ void raise_error(uint32_t *error_flag) {
    // with its result: the atomic has been performed when the wave goes on
    const uint32_t old = __hip_atomic_fetch_or(error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(old));
}

// ---- the row in LDS: 16 dwords per run, no padding.  The four 16-byte chunks of run r are
// stored in the order k ^ ((r >> 1) & 3), which spreads eight neighbouring runs over all 32
// banks for 16-byte accesses.  Every wave moves, reads and overwrites only the 4 KB of the row
// that its own lanes own (runs 64w .. 64w+63), so the row needs no workgroup barrier.
// (A row loaded straight into LDS, without the registers in between, does not pay here: the
// compiler makes every later LDS access of the wave wait for such a load, the reductions of
// the width search included.) ----
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
template <int B, int DT, bool FULL>
__device__ __forceinline__ void pack_to_image(const uint32_t (&m)[8], const Mags<DT> &mg, uint32_t *dst, uint32_t nd) {
    uint32_t o[8];
    {
        uint32_t t[B];
        pack_regs<B, DT>(m, mg, t);
#pragma unroll
        for (int k = 0; k < B; ++k) o[k] = t[k];
    }
    put_codes<B, FULL>(dst, o, nd);
}

// ---------------------------------------------------------------- the scanner (workgroup 0, one wave)

constexpr uint32_t kScanWavesMax = 4;   // waves of workgroup 0 that scan
// Groups of 64 table words per round.  A round takes about 1.8 us, so the window caps the tokens per second:
// 1024 tokens for the scanners of one to three waves (short rows, up to 300 tokens per us), 512 for four waves
// (rows of 8192 elements and more: at most 160 tokens per us; the smaller window polls fewer lines that the
// computing workgroups are writing to, which they notice)
constexpr int scan_groups(int waves) { return waves >= 4 ? 8 : 16; }

__device__ __forceinline__ uint64_t prefix_word(uint32_t tag, uint32_t ew, uint32_t ec) {
    return ((uint64_t)((tag << 30) | ew) << 32) | ec;
}

// The scanner: R waves of workgroup 0 (this one has index wv) work in rounds.  A round looks at
// the next 64 * scan_groups(R) tokens from the frontier on, cut into groups of 64 that are dealt out to
// the waves in turn (group k to wave k % R).  Every wave sums up its groups' leading runs of
// published tokens (lane l of a group is its l-th token: loads and stores are contiguous over
// the wave) and leaves their lengths and totals in LDS; after a barrier every wave knows, from
// those, which groups are usable (all before the first incomplete one, and that one up to its
// first gap) and what lies before each of its own, stores the prefixes of its groups, and moves
// the frontier, which all waves keep in step without exchanging it.
// lds: 8 + 2 * 3 * 16 dwords of LDS (workgroup 0 uses none otherwise).  waves_total: computing
// waves of the grid, each of which reports once when it is done.
template <int R>
__device__ void scan_tokens(const Params &p, uint8_t *blob, uint8_t *ws, uint32_t waves_total, uint32_t *lds,
                            uint32_t wv) {
    constexpr int kScanPerWave = scan_groups(R) / R;
    constexpr int kGroups = kScanPerWave * R;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t T = p.tokens, C = p.fused_classes;
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    uint32_t *sizes = reinterpret_cast<uint32_t *>(ws + p.ws_sizes);
    uint64_t *pre = reinterpret_cast<uint64_t *>(ws + p.ws_prefix);
    uint32_t *tickets = reinterpret_cast<uint32_t *>(ws + p.ws_tickets);
    uint64_t *pay_off = reinterpret_cast<uint64_t *>(blob + p.off_pay_off);
    uint64_t *row_ptr = reinterpret_cast<uint64_t *>(blob + p.off_row_ptr);
    uint32_t *error_flag = ctrl + kCtlError;
    __builtin_amdgcn_s_setprio(3);

    // a workspace that was reset for another shape (or never): nothing in it is touched, and the blob says so
    if (!workspace_shape_ok(uniform(word_load(ctrl + kCtlTokens + opaque_zero())),
                            uniform(word_load(ctrl + kCtlHidden + opaque_zero())), p.tokens, p.hidden)) {
        if (wv == 0 && lane == 0) write_header(p, blob, 0, 0, 5u);
        return;
    }
    const uint32_t epoch = (uniform(word_load(tickets + opaque_zero())) >> kTicketBits) % 3u;
    const uint32_t tag = epoch + 1u, tag3 = tag << 30;

    // Rows of a multiple of 32 elements (the common case) take H/32 payload words per bit of width, so
    // that one running sum serves both outputs: count + (width << 22) summed over 64 tokens carries
    // neither into the other (counts <= 2^15 each, widths <= 8).  Other rows get two sums.
    const bool packed = (p.hidden & 31u) == 0;
    const uint32_t words_per_bit = p.hidden >> 5;
    uint32_t pos = 0, bw = 0, bc = 0, idle = 0, round = 0;
    // wave 0 decides when to give up (its verdict travels with the round's data): a workspace that an
    // earlier call left in its failed state (or that was never reset) stays failed
    bool bad = wv == 0 && uniform(word_load(error_flag + opaque_zero())) != 0;
    while (pos < T) {
        uint32_t *lead_at = lds + 8 + (round & 1u) * 48u, *sum_at = lead_at + 16, *sum2_at = lead_at + 32;
        uint32_t w[kScanPerWave];
#pragma unroll
        for (int i = 0; i < kScanPerWave; ++i) {
            const uint32_t j = pos + 64u * (wv + (uint32_t)(R * i)) + lane;
            w[i] = 0;                                   // past the end: not published
            if (j < T) w[i] = word_load(sizes + j);
        }
        uint32_t before[kScanPerWave], before2[kScanPerWave], lead[kScanPerWave];
#pragma unroll
        for (int i = 0; i < kScanPerWave; ++i) {
            const uint64_t missing = __builtin_amdgcn_ballot_w64((w[i] & 0xC0000000u) != tag3);
            lead[i] = missing ? (uint32_t)__builtin_ctzll(missing) : 64u;     // published tokens in front of the group
            const bool mine = lane < lead[i];
            const uint32_t width = (w[i] >> 26) & 15u, cnt = w[i] & 0xFFFFu;
            uint32_t total, total2 = 0;
            if (packed) {
                const uint32_t v = mine ? cnt | (width << 22) : 0u;
                const uint32_t upto = wave_incl_scan_u32(v);
                before[i] = upto - v;
                before2[i] = 0;
                total = lane_value(upto, 63);
            } else {
                const uint32_t cw = mine ? row_bytes(p.hidden, width) >> 2 : 0u, cc = mine ? cnt : 0u;
                const uint32_t iw = wave_incl_scan_u32(cw), ic = wave_incl_scan_u32(cc);
                before[i] = ic - cc;
                before2[i] = iw - cw;
                total = lane_value(ic, 63);
                total2 = lane_value(iw, 63);
            }
            if (lane == 0) {
                const uint32_t k = wv + (uint32_t)(R * i);
                lead_at[k] = lead[i];
                sum_at[k] = total;
                sum2_at[k] = total2;
            }
        }
        if (wv == 0 && lane == 0) lds[0] = bad ? 1u : 0u;
        lds_barrier();
        if (uniform(lds[0])) { bad = true; break; }
        // ---- which groups count, and what lies before each: lane k looks at group k
        const uint32_t gl = lane < (uint32_t)kGroups ? lead_at[lane] : 64u;
        const uint64_t gaps = __builtin_amdgcn_ballot_w64(gl != 64u);
        const uint32_t first_gap = gaps ? (uint32_t)__builtin_ctzll(gaps) : (uint32_t)kGroups;   // groups before it are complete
        const bool counts = lane <= first_gap && lane < (uint32_t)kGroups;
        // (a packed group total is taken apart here: the widths of several groups would overflow their field)
        const uint32_t raw = counts ? sum_at[lane] : 0u;
        const uint32_t gs = packed ? raw & 0x3FFFFFu : raw;                                 // outliers of group `lane`
        const uint32_t gs2 = packed ? (raw >> 22) * words_per_bit : (counts ? sum2_at[lane] : 0u);   // its payload words
        const uint32_t upto = wave_incl_scan_u32(gs), upto2 = wave_incl_scan_u32(gs2);
        const uint32_t gone = wave_sum_u32(counts ? gl : 0u);                 // tokens the frontier moves by
#pragma unroll
        for (int i = 0; i < kScanPerWave; ++i) {
            const uint32_t k = wv + (uint32_t)(R * i);
            if (k <= first_gap && lane < lead[i]) {
                const uint32_t gb = lane_value(upto - gs, (int)k), gb2 = lane_value(upto2 - gs2, (int)k);
                // payload words / outliers before the lane's token
                const uint32_t ew = bw + gb2 + (packed ? (before[i] >> 22) * words_per_bit : before2[i]);
                const uint32_t ec = bc + gb + (packed ? before[i] & 0x3FFFFFu : before[i]);
                const uint32_t j = pos + 64u * k + lane;
                prefix_store(pre + j, prefix_word(tag, ew, ec));
                pay_off[j] = (uint64_t)ew << 2;
                row_ptr[j] = ec;
            }
        }
        bw += lane_value(upto2, 63);
        bc += lane_value(upto, 63);
        pos += gone;
        ++round;
        // nothing new for a long time: wave 0 gives up for everybody
        if (gone) idle = 0;
        else if (wv == 0 && !keep_waiting(idle, p.spin_limit, error_flag)) bad = true;
        else if (wv != 0) __builtin_amdgcn_s_sleep(2);
    }
    if (wv != 0) return;

    // ---- wave 0 closes the blob
    uint32_t spins = 0;
    if (!bad) {
        // every computing wave reports once, after its last store has been issued
        for (;;) {
            uint32_t v = 0;
            if (lane < C) v = word_load(tickets + lane * kTicketStride + kCntDone);
            const uint32_t done = wave_sum_u32(v);
            if (done == waves_total) break;
            if (!keep_waiting(spins, p.spin_limit, error_flag)) { bad = true; break; }
        }
    }
    if (!bad) bad = uniform(word_load(error_flag + opaque_zero())) != 0;
    if (bad) {
        if (lane == 0) {
            raise_error(error_flag);
            write_header(p, blob, 0, 0, 6u);
        }
        return;
    }
    // the counters as the next call expects them
    if (lane < kTicketClasses) {
        word_store(tickets + lane * kTicketStride + kCntDone, 0u);
        word_store(tickets + lane * kTicketStride + kCntTickets, ((epoch + 1u) % 3u) << kTicketBits);
    }
    if (lane == 0) {
        row_ptr[T] = bc;
        pay_off[T] = (uint64_t)bw << 2;
        write_header(p, blob, bc, (uint64_t)bw << 2, (uint64_t)bc > p.outlier_capacity ? 3u : 0u);
    }
}

// ---------------------------------------------------------------- computing workgroups

// One ticket of a class counter; the caller needs the result an iteration later.
__device__ __forceinline__ uint32_t draw_ticket(uint32_t *counter) {
    return __hip_atomic_fetch_add(counter + opaque_zero(), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What a wave keeps of a token between computing it and storing it (all uniform in the wave).
// Three words, not seven: the kernel is short of scalar registers, and what does not fit them is kept in lanes
// of a vector register and fetched back with a vector instruction at every use.
struct Pending {
    uint32_t token;
    uint32_t wpc;        // width | parity << 4 | outliers of the token << 8
    uint32_t split;      // outliers of the token in the waves before this one | those in this wave << 16
    __device__ __forceinline__ uint32_t width() const { return wpc & 15u; }
    __device__ __forceinline__ uint32_t parity() const { return (wpc >> 4) & 1u; }   // which payload image and stash hold it
    __device__ __forceinline__ uint32_t cnt() const { return wpc >> 8; }
    __device__ __forceinline__ uint32_t cb() const { return split & 0xFFFFu; }
    __device__ __forceinline__ uint32_t nw() const { return split >> 16; }
    __device__ __forceinline__ void set(uint32_t t, uint32_t width, uint32_t parity, uint32_t cnt, uint32_t cb, uint32_t nw) {
        token = t;
        wpc = width | (parity << 4) | (cnt << 8);
        split = cb | (nw << 16);
    }
};
struct Prefix {
    uint32_t ew, ec;     // payload words / outliers of all tokens before the token
    uint32_t bad;        // the wait expired
};

// Waits (bounded) until the scanner has published the prefix of `token`; v is what an earlier
// load of the entry returned.
__device__ __forceinline__ Prefix prefix_finish(const Params &p, const uint64_t *pre, uint32_t tag, uint32_t token,
                                                uint64_t v, uint32_t *error_flag) {
    uint32_t spins = 0;
    const uint64_t *at = pre + token + opaque_zero();
    while ((uint32_t)(v >> 62) != tag && keep_waiting(spins, p.spin_limit, error_flag)) v = prefix_load(at);
    Prefix x;
    x.bad = (uint32_t)(v >> 62) != tag ? 1u : 0u;
    x.ew = uniform((uint32_t)(v >> 32) & 0x3FFFFFFFu);
    x.ec = uniform((uint32_t)v);
    x.bad = uniform(x.bad);
    return x;
}

// Where a token's outputs go, and the LDS areas they come from.
struct StoreTargets {
    const Params &p;
    const uint16_t *in;
    uint32_t *payload;
    uint16_t *out_col, *out_val;
    const uint32_t *images, *stashes;
    uint32_t runs, pieces;
    uint32_t payload_words, outlier_capacity;      // both below 2^32: tokens * hidden is
};

// The lane's run of a token's row, read from memory again (see the rare case in store_wave_part).
__device__ __forceinline__ void reread_run(const StoreTargets &o, uint32_t token, uint32_t (&w)[16]) {
    const uint32_t r = threadIdx.x;                          // the lane's run
    const uint32_t have = 4u * r < o.pieces ? (o.pieces - 4u * r < 4u ? o.pieces - 4u * r : 4u) : 0u;
    const GlobalBytes src = (GlobalBytes)row_address(o.p, o.in, token, o.p.hidden) + 64u * r;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (k < have) v = *(const __attribute__((address_space(1))) u32x4 *)(src + 16u * k);
        w[4 * k] = v.x; w[4 * k + 1] = v.y; w[4 * k + 2] = v.z; w[4 * k + 3] = v.w;
    }
}

// Stores this wave's part of a token whose prefix is known: its 64 runs of the payload image
// LDS -> HBM (16 bytes per lane and step, contiguous over the wave) and its outliers from its
// stash.  Only what the wave wrote itself is read, so no barrier lies between this call and
// the writes.  Returns false without storing anything if the payload would leave its section,
// whatever the tables said.
// row_in_lds: the token's row is still in the LDS row buffer (the workgroup's last token).
// reread: the lane's run of the row as reread_run delivered it (asked for ahead of time), or null.
template <int DT, int NW>
__device__ __forceinline__ bool store_wave_part(const StoreTargets &o, const Pending &q, const Prefix &x,
                                                const uint32_t *row_in_lds = nullptr,
                                                const uint32_t (*reread)[16] = nullptr) {
    // the lane index through a register the compiler knows nothing about: the addresses derived
    // from it are computed here, not once before the token loop and then kept (or spilled) across it
    uint32_t lane = threadIdx.x & 63u;
    asm volatile("" : "+v"(lane));
    const uint32_t wv = uniform(threadIdx.x >> 6);
    const uint32_t width = q.width(), words = row_bytes(o.p.hidden, width) >> 2, nw = q.nw();
    if ((uint64_t)x.ew + words > (uint64_t)o.payload_words) return false;
    const uint32_t first = 64u * wv * width;                          // the wave's first dword of the image
    const uint32_t n = words > first ? (words - first < 64u * width ? words - first : 64u * width) : 0u;
    // Every address below is a uniform base (x is uniform) plus a byte offset of 32 bits: the base
    // stays in scalar registers and no lane holds a 64-bit pointer of its own.
    // (in the image every wave's codes start at its own fixed place, whatever the width: the regions
    // of two tokens of different widths never overlap between waves)
    const uint32_t *img = o.images + q.parity() * o.runs * 8u + wv * (64u * 8u);
    uint8_t *dst = reinterpret_cast<uint8_t *>(o.payload + x.ew + first);
    const uint32_t quads = n >> 2;            // at most 128: 8 bits x 32 elements per lane = 32 bytes
    const __amdgpu_buffer_rsrc_t window = raw_window(dst, n << 2);
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) {
        const uint32_t i = lane + r * 64u;
        if (i < quads) {
            // written through the L2 as it goes (the payload is what decompress reads next: it should stay
            // in the memory-side cache, which a streaming store would bypass; a plain store would leave
            // it dirty in the L2 until the end of the kernel, where writing it back costs about 2 us)
            const u32x4 v = *reinterpret_cast<const u32x4 *>(img + 4u * i);
            store_quad_through(window, 16u * i, v);
        }
    }
    const uint32_t rest = n & 3u;
    if (lane < rest) *reinterpret_cast<uint32_t *>(dst + 4u * (4u * quads + lane)) = img[4u * quads + lane];
    if (nw > 0 && (uint64_t)x.ec + q.cnt() <= (uint64_t)o.outlier_capacity) {
        uint8_t *col = reinterpret_cast<uint8_t *>(o.out_col + x.ec + q.cb());
        uint8_t *val = reinterpret_cast<uint8_t *>(o.out_val + x.ec + q.cb());
        if (nw <= kStashWave) {
            const uint32_t *stash = o.stashes + (q.parity() * NW + wv) * kStashWave;
            for (uint32_t k = lane; k < nw; k += 64u) {
                const uint32_t e = stash[k];
                *reinterpret_cast<uint16_t *>(col + 2u * k) = (uint16_t)(e >> 16);
                *reinterpret_cast<uint16_t *>(val + 2u * k) = (uint16_t)e;
            }
        } else {
            // rare: more outliers than the wave's stash holds, so none was kept.  The wave takes its part
            // of the row once more (from LDS if it is still there, else from memory: it is two
            // iterations old and still in the caches), splits it again and stores the outliers out of
            // the registers, in column order.
            const uint32_t r = 64u * wv + lane;                  // the lane's run
            const uint32_t have = 4u * r < o.pieces ? (o.pieces - 4u * r < 4u ? o.pieces - 4u * r : 4u) : 0u;
            uint32_t w[16];
            if (row_in_lds) {
                load_run_sw(row_in_lds, have ? r : 0u, w);       // pieces beyond the row were written as zeros
                if (!have) {
#pragma unroll
                    for (int k = 0; k < 16; ++k) w[k] = 0;
                }
            } else if (reread) {
#pragma unroll
                for (int k = 0; k < 16; ++k) w[k] = (*reread)[k];
            } else {
                reread_run(o, q.token, w);
            }
            Mags<DT> unused;
            uint32_t omask = 0, amax_bits = 0;
            split_regs<DT, false>(w, o.p.thr_pk, unused, omask, amax_bits);
            const uint32_t nl = (uint32_t)__builtin_popcount(omask);
            uint32_t pos = 2u * (wave_incl_scan_u32(nl) - nl);       // bytes into the wave's CSR slice
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (omask & (1u << (2 * i))) {
                    *reinterpret_cast<uint16_t *>(col + pos) = (uint16_t)(32u * r + 2u * i);
                    *reinterpret_cast<uint16_t *>(val + pos) = (uint16_t)w[i];
                    pos += 2u;
                }
                if (omask & (2u << (2 * i))) {
                    *reinterpret_cast<uint16_t *>(col + pos) = (uint16_t)(32u * r + 2u * i + 1u);
                    *reinterpret_cast<uint16_t *>(val + pos) = (uint16_t)(w[i] >> 16);
                    pos += 2u;
                }
            }
        }
    }
    return true;
}

// LDS map (dynamic): row: runs*16 | two payload images: runs*8 each | ring: 4 reduce areas |
// ticket slots (8 dwords) | stashes: 2 x NW x kStashWave dwords
constexpr uint32_t kLdsRing = 4 * 2 * kMaxWaves;
static_assert(kFusedScratchDw == kLdsRing + 8, "LDS map of the fused kernel");

// Row t of the input: one tensor, or (BATCH) a device table of tensor pointers, rows_per_tensor rows each.
template <bool BATCH>
__device__ __forceinline__ const uint16_t *input_row(const Params &p, const uint16_t *in, uint32_t t, uint32_t hidden) {
    if (!BATCH) return in + (size_t)t * hidden;
    return row_address(p, in, t, hidden);
}

// FULL: the row fills the workgroup exactly (hidden == 2048 * NW), so every lane owns a whole run
// and none of the range checks of the general case is needed.
template <int DT, int NW, bool FULL, bool BATCH>
__global__ void __launch_bounds__(64 * NW, 4)
k_fused(const Params p, const uint16_t *__restrict__ in, uint8_t *__restrict__ blob, uint8_t *__restrict__ ws) {
    extern __shared__ __align__(16) uint32_t lds[];
    if (blockIdx.x == 0) {
        constexpr int kScanWaves = NW < (int)kScanWavesMax ? NW : (int)kScanWavesMax;
        if (threadIdx.x < 64u * kScanWaves)
            scan_tokens<kScanWaves>(p, blob, ws, (gridDim.x - 1u) * NW, lds, threadIdx.x >> 6);
        return;
    }
    uint32_t *lrow = lds;
    const uint32_t runs = FULL ? 64u * NW : p.runs, pieces = FULL ? 256u * NW : p.pieces;
    uint32_t *images = lds + runs * 16u;                    // packed codes of the current and the pending token
    uint32_t *ring = images + 2u * runs * 8u;
    uint32_t *tslot = ring + kLdsRing;                      // next token, one slot per iteration parity; first token, epoch
    uint32_t *stashes = tslot + 8;                          // 2 x NW x kStashWave dwords: col << 16 | raw value
    const uint32_t tid = threadIdx.x, run = tid;
    const uint32_t wg = blockIdx.x - 1u;
    const uint32_t wv = uniform(tid >> 6);
    const bool owns = FULL || run < runs;
    const uint32_t left = FULL ? 4u : (owns ? pieces - 4 * run : 0);   // 16-byte pieces of the lane's run inside the row

    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    uint32_t *error_flag = ctrl + kCtlError;
    uint32_t *sizes = reinterpret_cast<uint32_t *>(ws + p.ws_sizes);
    const uint64_t *pre = reinterpret_cast<const uint64_t *>(ws + p.ws_prefix);

    // ticket class of this workgroup: class c owns the tokens t % C == c
    const uint32_t C = p.fused_classes, cls = wg % C;
    const uint32_t n_cls = (p.tokens - cls + C - 1u) / C;   // tokens of the class (cls < C <= G <= tokens)
    uint32_t *counter = reinterpret_cast<uint32_t *>(ws + p.ws_tickets) + cls * kTicketStride;

    uint8_t *bits = blob + p.off_bits;
    float *scale = reinterpret_cast<float *>(blob + p.off_scale);
    uint16_t *out_col = reinterpret_cast<uint16_t *>(blob + p.off_out_col);
    uint16_t *out_val = reinterpret_cast<uint16_t *>(blob + p.off_out_val);
    const uint32_t hidden = FULL ? 2048u * NW : p.hidden;

    // ---- the first ticket: this workgroup's first token
    if (tid == 0) {
        // (the counters lie at the same place in every workspace; the ticket is drawn while the shape is
        // on its way, and handed back if the workspace turns out to be another plan's or never reset: the
        // scanner reports that, and the workspace is left as it was)
        const uint32_t first = draw_ticket(counter);
        const uint32_t ws_tokens = word_load(ctrl + kCtlTokens + opaque_zero());
        const uint32_t ws_hidden = word_load(ctrl + kCtlHidden + opaque_zero());
        if (workspace_shape_ok(ws_tokens, ws_hidden, p.tokens, p.hidden)) {
            const uint32_t k = first & kTicketMask;
            tslot[2] = k < n_cls ? k * C + cls : kNoToken;
            tslot[3] = (first >> kTicketBits) % 3u + 1u;
        } else {
            __hip_atomic_fetch_sub(counter + opaque_zero(), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            tslot[2] = kNoToken;
            tslot[3] = 0;
        }
    }
    __syncthreads();
    uint32_t t = uniform(tslot[2]);
    const uint32_t tag = uniform(tslot[3]);
    if (tag == 0) return;

    // the row of the next iteration on its way HBM -> registers -> LDS (each wave its own part)
    RowPart pre_row;
    if (t != kNoToken) {
        fetch_row_part<FULL>(reinterpret_cast<const uint4 *>(input_row<BATCH>(p, in, t, hidden)), pieces, pre_row);
        write_row_part_sw<FULL>(lrow, runs, pre_row);
    }

    uint32_t failed = 0, turn = 0;         // turn: rotation through the reduce areas
    // tokens computed but not stored yet: `young` is from the previous iteration, `old` from the one
    // before.  A token's payload image and stash are those of its iteration's parity, so `old` has
    // to leave before the current token's codes are packed into the same image.
    Pending young, old;
    bool have_young = false, have_old = false;
    young.set(0, 8, 0, 0, 0, 0);
    old = young;

    const StoreTargets out{p, in, reinterpret_cast<uint32_t *>(blob + p.off_payload), out_col, out_val, images, stashes,
                           runs, pieces, as_computed((uint32_t)(p.payload_capacity >> 2)), as_computed((uint32_t)p.outlier_capacity)};

    // The end of a call: workgroups that were dispatched later run slower (the instruction arbiter of
    // a SIMD prefers its older waves), and whoever starts a token among the last ones keeps everybody
    // waiting for it.  So the later half of the workgroups stops drawing tickets a little before the
    // tokens run out (the last quarter 1.25 generations before, the third quarter half a generation
    // before; a generation = one token per workgroup) and leaves the rest to the faster ones, which then
    // have their compute units more to themselves.  Only for calls of at least six generations, and
    // never for the first quarter of a class, so every token is still drawn.
    uint32_t kmine = t != kNoToken ? (t - cls) / C : 0u;     // thread 0: the class's number of the workgroup's newest token
    const uint32_t n_wg = gridDim.x - 1u, w_cls = (n_wg - cls + C - 1u) / C;
    const uint32_t quarter = n_wg >= 4u * C && n_cls >= 6u * w_cls ? (4u * wg) / n_wg : 0u;
    const uint32_t stop_margin = (w_cls * (quarter == 3u ? 5u : quarter == 2u ? 2u : 0u)) / 4u;
    uint32_t it = 0;
    for (; t != kNoToken; ++it) {
        // ---- the ticket of the token after this one: drawn now, taken after the threshold split.  A
        //      workgroup holds one token beyond the one it works on, no more, so that the last tokens of
        //      a call spread evenly over the workgroups.
        uint32_t req = 0;
        if (tid == 0) {
            if (n_cls - 1u - kmine < stop_margin) req = kTicketMask;       // leave the last tokens to the faster workgroups
            else req = draw_ticket(counter);
        }

        // ---- Eq. (ts) for token t
        Mags<DT> mg;
        uint32_t omask = 0, amax_bits = 0;
        {
            uint32_t w[16];
            load_run_sw(lrow, owns ? run : 0u, w);
            split_regs<DT, true>(w, p.thr_pk, mg, omask, amax_bits);
        }
        if (!owns) { omask = 0; amax_bits = 0; }

        // outliers of the token in this wave, and before each lane
        const uint32_t nl = (uint32_t)__builtin_popcount(omask);
        const uint32_t upto = wave_incl_scan_u32(nl);               // outliers of the wave's lanes up to this one
        const uint32_t cnt_wave = lane_value(upto, 63);
        // (the ticket is taken here and not earlier: the empty statement ties its first use to a result of
        // the split, or the wait for it would be placed right behind the draw)
        asm volatile("" : "+v"(req) : "v"(upto));
        if (tid == 0) {
            const uint32_t k = req & kTicketMask;
            tslot[it & 1u] = k < n_cls ? k * C + cls : kNoToken;      // read behind the barrier of the reduction
            kmine = k;
        }

        // ---- Algorithm 1.  The width search is where the waves of a workgroup meet at barriers (one per
        // cross-wave reduction).  A compute unit's SIMDs each hold one wave of several workgroups; with the
        // waves of the workgroup that is in this phase preferred by the instruction arbiter, they reach
        // each barrier together instead of each being held up by whatever its SIMD's other waves
        // happen to do, and less time is lost waiting there.
        __builtin_amdgcn_s_setprio(1);
        const RowStats st = reduce_row_stats_counted<NW>(amax_bits, cnt_wave, ring, turn);
        const uint32_t tn = uniform(tslot[it & 1u]);
        // the prefix of the older pending token: asked for now (as late as it can be and still arrive
        // behind the width search), used after the search
        uint64_t early = 0;
        if (have_old) early = prefix_load(pre + old.token + opaque_zero());
        // The next row starts its way from HBM (into registers; it goes to LDS at the end of the
        // iteration).  The loads are issued on every path (without a next token every lane reads the first
        // piece of the current row, which costs one cache line), so that the number of loads younger than
        // the prefix load is fixed and waiting for the prefix below does not wait for the row.
        fetch_row_part<FULL>(reinterpret_cast<const uint4 *>(input_row<BATCH>(p, in, tn != kNoToken ? tn : t, hidden)),
                             pieces, pre_row, tn != kNoToken ? 16u : 0u);
        uint32_t m[8];
        const Choice c = search_width<DT, NW>(p, mg, st.amax, owns, ring, turn, m);
        __builtin_amdgcn_s_setprio(0);
        // the prefix asked for at the top: taken as late as the stores allow
        Prefix xo;
        xo.ew = xo.ec = xo.bad = 0;
        if (have_old) xo = prefix_finish(p, pre, tag, old.token, early, error_flag);
        if (tid == 0) {
            word_store(sizes + t, (tag << 30) | (c.width << 26) | st.cnt);
            bits[t] = (uint8_t)c.width;
            scale[t] = c.scale;
        }

        // ---- store this wave's part of the token of two iterations ago: its image and stash are needed now
        if (have_old) {
            if (xo.bad || !store_wave_part<DT, NW>(out, old, xo)) failed = 1;
            have_old = false;
        }

        // ---- codes of the lane's run at the chosen width, into this iteration's payload image
        Pending cur;
        cur.set(t, c.width, it & 1u, st.cnt, st.cnt_before, cnt_wave);
        if (owns) {
            uint32_t *dst = images + (it & 1u) * runs * 8u + wv * (64u * 8u) + (run & 63u) * c.width;
            const uint32_t nd = (FULL || left >= 4) ? c.width : ((left * c.width + 3u) >> 2);
            switch (c.width) {
                case 2: pack_to_image<2, DT, FULL>(m, mg, dst, nd); break;
                case 3: pack_to_image<3, DT, FULL>(m, mg, dst, nd); break;
                case 4: pack_to_image<4, DT, FULL>(m, mg, dst, nd); break;
                case 5: pack_to_image<5, DT, FULL>(m, mg, dst, nd); break;
                case 6: pack_to_image<6, DT, FULL>(m, mg, dst, nd); break;
                case 7: pack_to_image<7, DT, FULL>(m, mg, dst, nd); break;
                default: pack_to_image<8, DT, FULL>(m, mg, dst, nd); break;
            }
        }
        // ---- T_above of token t, this wave's part: into the wave's stash of this parity (free since the
        //      store above) in column order; a wave with more outliers than its stash holds keeps
        //      nothing (see store_wave_part)
        if (cnt_wave > 0 && cnt_wave <= kStashWave) {
            uint32_t *stash = stashes + ((it & 1u) * NW + wv) * kStashWave;
            uint32_t pos = upto - nl;
            for (uint32_t rest = omask; rest; rest &= rest - 1u) {
                const uint32_t j = (uint32_t)__builtin_ctz(rest);
                stash[pos++] = ((run * kRun + j) << 16) | raw_element_sw(lrow, run, j);
            }
        }
        old = young; have_old = have_young;
        young = cur; have_young = true;
        if (tn != kNoToken) write_row_part_sw<FULL>(lrow, runs, pre_row);   // this wave is done with its part of the row
        t = tn;
    }

    // ---- the tokens still pending, oldest first (both prefixes are asked for at once)
    uint64_t last_old = 0, last_young = 0;
    if (have_old) last_old = prefix_load(pre + old.token + opaque_zero());
    if (have_young) last_young = prefix_load(pre + young.token + opaque_zero());
    // (a wave that kept none of the older token's outliers asks for its part of that row now, not
    // when the prefix has arrived)
    uint32_t again[16];
    const bool old_reread = have_old && old.nw() > kStashWave;
    if (old_reread) reread_run(out, old.token, again);
    if (have_old) {
        const Prefix x = prefix_finish(p, pre, tag, old.token, last_old, error_flag);
        if (x.bad || !store_wave_part<DT, NW>(out, old, x, nullptr, old_reread ? &again : nullptr)) failed = 1;
    }
    if (have_young) {
        // the row of the workgroup's last token was not overwritten by a next one
        const Prefix x = prefix_finish(p, pre, tag, young.token, last_young, error_flag);
        if (x.bad || !store_wave_part<DT, NW>(out, young, x, lrow)) failed = 1;
    }
    // ---- this wave is done
    if ((tid & 63u) == 0) {
        if (failed) raise_error(error_flag);
        __hip_atomic_fetch_add(counter + kCntDone + opaque_zero(), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------- launchers

static hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

typedef void (*FusedKernel)(const Params, const uint16_t *, uint8_t *, uint8_t *);

template <int DT, bool FULL, bool BATCH>
static FusedKernel fused_kernel_for(uint32_t nw) {
    switch (nw) {
        case 1: return k_fused<DT, 1, FULL, BATCH>;
        case 2: return k_fused<DT, 2, FULL, BATCH>;
        case 3: return k_fused<DT, 3, FULL, BATCH>;
        case 4: return k_fused<DT, 4, FULL, BATCH>;
        case 8: return k_fused<DT, 8, FULL, BATCH>;
        default: return k_fused<DT, 16, FULL, BATCH>;
    }
}
template <int DT>
static FusedKernel fused_kernel_dt(uint32_t nw, bool full, bool batch) {
    if (full) return batch ? fused_kernel_for<DT, true, true>(nw) : fused_kernel_for<DT, true, false>(nw);
    return batch ? fused_kernel_for<DT, false, true>(nw) : fused_kernel_for<DT, false, false>(nw);
}
static FusedKernel fused_kernel(uint32_t dtype, uint32_t nw, bool full, bool batch) {
    return dtype == (uint32_t)kF16 ? fused_kernel_dt<kF16>(nw, full, batch) : fused_kernel_dt<kBF16>(nw, full, batch);
}
static bool fills_workgroup(const Params &p, const Geometry &g) { return p.hidden == 2048u * g.waves; }

// waves per workgroup of the fused kernel for a row of `runs` runs: the smallest instantiated size
uint32_t compress_waves(uint32_t runs) {
    const uint32_t need = (runs + 63u) / 64u;
    if (need <= 4) return need;
    return need <= 8 ? 8u : 16u;
}

int prepare_fused_kernels() {
    const int big = (int)(((kMaxHidden / kRun) * 32u + kFusedScratchDw + 2u * kMaxWaves * kStashWave) * 4);
    static const uint32_t sizes[] = {1, 2, 3, 4, 8, 16};
    for (uint32_t dt = 0; dt < 2; ++dt)
        for (uint32_t nw : sizes)
            for (int v = 0; v < 4; ++v) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fused_kernel(dt, nw, (v & 1) != 0, (v & 2) != 0)),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, big);
                if (e != hipSuccess) return (int)e;
            }
    return 0;
}

// Workgroups of this plan's kernel that the current device holds at once.  The answer depends on
// the device, the kernel and its LDS size only; it is looked up once per such combination.
int fused_resident_workgroups(const Params &p, const Geometry &g, uint32_t *out) {
    struct Entry { int dev; const void *fn; uint32_t lds; uint32_t resident; };
    static std::mutex mutex;
    static Entry cache[64];
    static int used = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    const void *fn = reinterpret_cast<const void *>(fused_kernel(p.dtype, g.waves, fills_workgroup(p, g), p.rows_per_tensor != 0));
    std::lock_guard<std::mutex> lock(mutex);
    for (int i = 0; i < used; ++i)
        if (cache[i].dev == dev && cache[i].fn == fn && cache[i].lds == g.lds_fused_bytes) {
            *out = cache[i].resident;
            return 0;
        }
    int cus = 0, per_cu = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, (int)(64u * g.waves), g.lds_fused_bytes);
    if (e != hipSuccess) return (int)e;
    if (per_cu < 1 || cus < 1) return (int)hipErrorInvalidConfiguration;
    *out = (uint32_t)per_cu * (uint32_t)cus;
    if (used < 64) cache[used++] = Entry{dev, fn, g.lds_fused_bytes, *out};
    return 0;
}

// grid: computing workgroups (the scanner is added here)
int launch_fused(const Params &p, const Geometry &g, uint32_t grid, const void *d_in, void *d_blob, void *d_ws,
                 void *stream) {
    hipLaunchKernelGGL(fused_kernel(p.dtype, g.waves, fills_workgroup(p, g), p.rows_per_tensor != 0), dim3(grid + 1u),
                       dim3(64u * g.waves),
                       g.lds_fused_bytes, as_stream(stream), p, static_cast<const uint16_t *>(d_in),
                       static_cast<uint8_t *>(d_blob), static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------- workspace reset

__global__ void k_ws_reset(const Params p, uint8_t *__restrict__ ws) {
    uint32_t *sizes = reinterpret_cast<uint32_t *>(ws + p.ws_sizes);
    uint32_t *pre = reinterpret_cast<uint32_t *>(ws + p.ws_prefix);
    uint32_t *tickets = reinterpret_cast<uint32_t *>(ws + p.ws_tickets);
    uint32_t *ctrl = reinterpret_cast<uint32_t *>(ws + p.ws_ctrl);
    const uint32_t stride = gridDim.x * blockDim.x, first = blockIdx.x * blockDim.x + threadIdx.x;
    for (uint32_t i = first; i < p.tokens; i += stride) sizes[i] = 0;
    for (uint64_t i = first; i < 2ull * (p.tokens + 1ull); i += stride) pre[i] = 0;
    for (uint32_t i = first; i < kTicketClasses * kTicketStride; i += stride) tickets[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x < 64)
        ctrl[threadIdx.x] = threadIdx.x == kCtlTokens ? p.tokens : threadIdx.x == kCtlHidden ? p.hidden : 0u;
}

int launch_ws_reset(const Params &p, void *d_ws, void *stream) {
    uint32_t blocks = (p.tokens + 255u) / 256u;
    if (blocks < 32) blocks = 32;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_ws_reset, dim3(blocks), dim3(256), 0, as_stream(stream), p, static_cast<uint8_t *>(d_ws));
    return (int)hipGetLastError();
}

}  // namespace tsq
