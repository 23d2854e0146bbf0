// Entropy coding of the packed codes (gfx950): the rANS stage that the paper places after TAB-Q
// (Sec. II-C.2, last paragraph).  The paper leaves the coder to a third-party package; format and
// kernels here are this library's own.
//
// Format.  One frequency table per width class (all tokens of one width share it): pooled code
// counts scaled to 12 bits.  Every token is coded on its own by 64 interleaved rANS coders, one
// per lane of a wave (state in [2^16, 2^32), 16-bit renormalisation).  The token's codes are cut
// into runs of 32, as everywhere in this library; coder l owns the runs l, l + 64, ...; step i
// handles element i % 32 of run number i / 32 of every coder.  The encoder walks the steps
// backwards, the decoder forwards; the 16-bit words that the coders shed in one step are stored
// in lane order (a ballot and a population count give every lane its place).  A token's stream
// is the final states of the coders that own a run (min(64, runs) of them) followed by the words
// in the order the decoder reads them, padded to 4 bytes.
//
// Encode: code counts per width, added to one of 16 sets (k_code_pool) -> sets added up,
// tables (k_rans_tables) -> one wave per token codes its stream into a slot of the workspace
// (k_rans_encode) and adds its length to the stream bytes of its block of 256 tokens -> every token
// finds its offset from the block sums before it and the lengths before it inside its block, and its
// stream moves to its place (k_rans_gather).
// Decode: one wave per token (k_rans_decode) rebuilds the packed payload; the words it reads
// pass through registers (windows of 64 words), so a token needs 5 KB of LDS for its tables
// and nothing else, and a compute unit holds its full 32 waves.
#include <hip/hip_runtime.h>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

constexpr uint32_t kProbBits = 12, kProbScale = 1u << kProbBits, kRansLow = 1u << 16;
static_assert(kProbScale == 4096, "frequency_slot() masks 12 bits");

__device__ __forceinline__ bool blob_is_valid(const Params &p, const uint8_t *blob) {
    const BlobHeader *h = reinterpret_cast<const BlobHeader *>(blob);
    return h->magic == kMagic && h->version == kVersion && h->status == 0 && h->tokens == p.tokens &&
           h->hidden == p.hidden && h->dtype == p.dtype && h->off_payload == p.off_payload;
}
__device__ __forceinline__ bool eblob_is_valid(const Params &p, const EntropyLayout &e, const uint8_t *eblob) {
    const EntropyHeader *h = reinterpret_cast<const EntropyHeader *>(eblob);
    return h->magic == kEntropyMagic && h->version == kVersion && h->tokens == p.tokens && h->hidden == p.hidden &&
           h->off_streams == e.off_streams && h->stream_bytes <= e.stream_capacity;
}

// ---------------------------------------------------------------- pooled counts and tables

// What the kernels of a call add to starts at zero: the pooled code counts and the stream bytes per block of
// tokens (one thread per word).
constexpr uint32_t kBeginThreads = 1024;
__global__ void __launch_bounds__(kBeginThreads)
k_rans_begin(const Params p, const EntropyLayout e, uint8_t *__restrict__ eblob, uint8_t *__restrict__ ews) {
    const uint32_t i = blockIdx.x * kBeginThreads + threadIdx.x, n_counts = kPoolCopies * 7u * 256u;
    const uint32_t n_blocks = (p.tokens + kLenBlock - 1u) / kLenBlock;
    if (i < n_counts) reinterpret_cast<uint32_t *>(ews + e.ws_pooled)[i] = 0;
    else if (i - n_counts < n_blocks) reinterpret_cast<uint32_t *>(ews + e.ws_block)[(i - n_counts) * kBlockStride] = 0;
    // the header becomes valid only when the last kernel of the call has run
    if (blockIdx.x == 0 && threadIdx.x < sizeof(EntropyHeader) / 4) reinterpret_cast<uint32_t *>(eblob)[threadIdx.x] = 0;
}

// One workgroup per width class: counts -> 12-bit frequencies.  f_c = max(1, floor(n_c * 4096 / N))
// for n_c > 0; while the sum exceeds 4096, one is taken from the largest f (lowest code on ties);
// a remaining deficit goes to the code with the largest count (lowest code on ties).
// Taking E times one from the current largest entry is a cut at a level: with
// g(v) = sum_c max(f_c - v, 0), the level is the v with g(v + 1) < E <= g(v); every entry above
// v + 1 comes down to v + 1, and the first E - g(v + 1) entries (in code order) that then stand at
// v + 1 go down to v.  The level is found by bisection, each probe a workgroup-wide sum.
__global__ void __launch_bounds__(256)
k_rans_tables(const Params p, const EntropyLayout e, const uint8_t *__restrict__ blob, uint8_t *__restrict__ eblob,
              const uint8_t *__restrict__ ews) {
    __shared__ uint32_t part[3][4];
    if (!blob_is_valid(p, blob)) return;
    const uint32_t k = blockIdx.x, c = threadIdx.x;
    // this class's counts: the sets that the counting workgroups added to, added up
    const uint32_t *counts = reinterpret_cast<const uint32_t *>(ews + e.ws_pooled) + k * 256u;
    uint16_t *table = reinterpret_cast<uint16_t *>(eblob + e.off_tables) + k * 256u;
    // workgroup-wide sum of one value per thread: wave sums, exchanged through one of three areas in
    // rotation (an area is written again two barriers after it was read), one barrier per sum
    uint32_t turn = 0;
    auto block_sum = [&](uint32_t v) {
        uint32_t *area = part[turn % 3u];
        ++turn;
        const uint32_t w = wave_sum_u32(v);
        if ((c & 63u) == 0) area[c >> 6] = w;
        __syncthreads();
        return area[0] + area[1] + area[2] + area[3];
    };
    auto block_max = [&](uint32_t v) {
        uint32_t *area = part[turn % 3u];
        ++turn;
        const uint32_t w = wave_max_u32(v);
        if ((c & 63u) == 0) area[c >> 6] = w;
        __syncthreads();
        const uint32_t a = area[0] > area[1] ? area[0] : area[1], b = area[2] > area[3] ? area[2] : area[3];
        return a > b ? a : b;
    };
    uint32_t nc = 0;
#pragma unroll
    for (uint32_t g = 0; g < kPoolCopies; ++g) nc += counts[g * 7u * 256u + c];
    const uint32_t N = block_sum(nc);
    uint32_t fc = 0;
    if (N && nc) {
        fc = (uint32_t)(((uint64_t)nc << kProbBits) / N);
        if (fc == 0) fc = 1;
    }
    const uint32_t S = block_sum(fc);
    if (S > kProbScale) {
        const uint32_t E = S - kProbScale;
        uint32_t lo = 0, hi = kProbScale;        // g(lo) >= E always (g(0) = S > E); g(hi) = 0 < E
        while (hi - lo > 1u) {                   // invariant: g(lo) >= E > g(hi)
            const uint32_t mid = (lo + hi) >> 1;
            const uint32_t g = block_sum(fc > mid ? fc - mid : 0u);
            if (g >= E) lo = mid; else hi = mid;
        }
        // level lo: g(lo + 1) < E <= g(lo)
        const uint32_t above = block_sum(fc > lo + 1u ? fc - (lo + 1u) : 0u);
        const uint32_t rest = E - above;         // entries at lo + 1 (after the cut) that go one further down
        // rank of this code among those above the level, in code order: lanes below in the wave, waves before
        const uint64_t mine = __builtin_amdgcn_ballot_w64(fc > lo);
        uint32_t *area = part[turn % 3u];
        ++turn;
        if ((c & 63u) == 0) area[c >> 6] = (uint32_t)__builtin_popcountll(mine);
        __syncthreads();
        uint32_t rank = (uint32_t)__builtin_popcountll(mine & ((1ull << (c & 63u)) - 1ull));
        for (uint32_t w = 0; w < (c >> 6); ++w) rank += area[w];
        if (fc > lo) fc = rank < rest ? lo : lo + 1u;
    } else if (N && S < kProbScale) {
        // the lowest code among those with the largest count: the largest of 256 - c over them
        const uint32_t most = block_max(nc);
        const uint32_t pick = block_max(nc == most ? 256u - c : 0u);
        if (256u - c == pick) fc += kProbScale - S;
    }
    table[c] = (uint16_t)fc;
}

// The table of a token's class into LDS, by one wave (lane l owns the codes 4l .. 4l+3): per code
// x = f | cum << 16 (cum = exclusive running sum, < 4096) and y = the binary32 pattern of a value a
// little below 1 / f (see quotient_or_one_less).  Eight bytes per code: wider entries cost more LDS
// time than the instructions they save.
// A code the table does not know (f = 0; cannot happen for a table built from the blob that is
// coded) is entered with f = 1, which keeps the division defined.
__device__ __forceinline__ void load_table(const uint16_t *table, uint2 *ftab) {
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t f[4], s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[i] = table[4u * lane + i]; s += f[i]; }
    uint32_t cum = wave_incl_scan_u32(s) - s;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t fi = f[i] ? f[i] : 1u;
        ftab[4u * lane + i] = make_uint2(fi | (cum << 16), __float_as_uint(reciprocal_just_below(fi)));
        cum += f[i];
    }
}

// The decoder's form of the table: f | cum << 16 only (it never divides), 1 KB, so that a token's
// tables take 5 KB of LDS and a compute unit holds 32 tokens at once.  Unknown codes keep f = 0.
__device__ __forceinline__ void load_table_decode(const uint16_t *table, uint32_t *ftab) {
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t f[4], s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[i] = table[4u * lane + i]; s += f[i]; }
    uint32_t cum = wave_incl_scan_u32(s) - s;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ftab[4u * lane + i] = f[i] | (cum << 16);
        cum += f[i];
    }
}

// How many of the lanes before this one are set in `who`.
__device__ __forceinline__ uint32_t rank_in(uint64_t who) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(who >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)who, 0u));
}

// ---------------------------------------------------------------- encode

// The steps of one round (run number `round` of every lane), last element first.  The words go
// straight to the token's slot in the workspace, which fills from its end downwards.
// WHOLE: every lane's run of this round lies inside the row (valid >= 32 everywhere), so no step
// needs a range check.
template <int B, bool WHOLE>
__device__ __forceinline__ void encode_round(const uint32_t *src_row, uint32_t run, int valid, const uint2 *ftab,
                                             uint16_t *out, uint32_t &ptr, uint32_t &x) {
    uint32_t d[B];
    const uint32_t nd = (WHOLE || valid >= 32) ? (uint32_t)B : (valid > 0 ? ((uint32_t)valid * B + 31u) >> 5 : 0u);
    if (WHOLE) {
        load_run_words<B>(src_row + run * B, d);
    } else {
#pragma unroll
        for (int k = 0; k < B; ++k) d[k] = (uint32_t)k < nd ? src_row[run * B + k] : 0u;
    }
#pragma unroll
    for (int j = 31; j >= 0; --j) {
        const int off = j * B, k = off >> 5, sh = off & 31;
        uint32_t code = d[k] >> sh;
        if (sh + B > 32) code |= d[k + 1 < B ? k + 1 : k] << (32 - sh);
        code &= (1u << B) - 1u;
        const bool active = WHOLE || j < valid;
        const uint2 entry = ftab[code];
        const uint32_t f = entry.x & 0xFFFFu;
        const bool shed = active && (x >> 20) >= f;            // x >= f << 20, without overflow for f = 4096
        const uint64_t who = __builtin_amdgcn_ballot_w64(shed);
        ptr -= (uint32_t)__builtin_popcountll(who);
        if (shed) {
            // (a 32-bit byte offset from a uniform base: one instruction for the address)
            const uint32_t at = (ptr + rank_in(who)) << 1;
            *reinterpret_cast<uint16_t *>(reinterpret_cast<uint8_t *>(out) + at) = (uint16_t)x;
            x >>= 16;
        }
        if (active) {
            // x -> (q << 12) + (x - q f) + cum with q = floor(x / f) = q1 or q1 + 1
            const uint32_t q1 = quotient_or_one_less(x, __uint_as_float(entry.y));
            const uint32_t r1 = x - __umul24(q1, f);           // x - q1 f: the remainder, or f more
            const uint32_t more = r1 >= f ? kProbScale - f : 0u;
            x = (q1 << kProbBits) + r1 + (entry.x >> 16) + more;
        }
    }
}

// Slot of a token in the workspace: room for 64 states (256 bytes), then room for one word per element of
// the padded row; the words stand at the END of that room (the encoder fills it backwards).
__global__ void __launch_bounds__(64)
k_rans_encode(const Params p, const EntropyLayout e, const uint8_t *__restrict__ blob, const uint8_t *__restrict__ eblob,
              uint8_t *__restrict__ ews) {
    __shared__ uint2 ftab[256];
    const uint32_t t = blockIdx.x, lane = threadIdx.x;
    uint32_t *len = reinterpret_cast<uint32_t *>(ews + e.ws_len);
    if (!blob_is_valid(p, blob)) return;
    const uint32_t width = blob[p.off_bits + t];
    const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
    if (!token_in_range(p, width, po)) {
        if (lane == 0) len[t] = 0;
        return;
    }
    load_table(reinterpret_cast<const uint16_t *>(eblob + e.off_tables) + (width - 2u) * 256u, ftab);
    __syncthreads();
    const uint32_t *src_row = reinterpret_cast<const uint32_t *>(blob + p.off_payload + po);
    uint8_t *slot = ews + e.ws_slots + (size_t)t * e.slot_bytes;
    uint16_t *out = reinterpret_cast<uint16_t *>(slot + 256);
    const uint32_t rounds = (p.runs + 63u) / 64u, cap = (e.slot_bytes - 256u) >> 1;   // one word per element at most
    uint32_t x = kRansLow, ptr = cap;
    for (uint32_t r = rounds; r-- > 0;) {
        const uint32_t run = lane + 64u * r;
        const int valid = (int)p.hidden - (int)(run * kRun);          // may be <= 0: nothing of this run exists
        if (__builtin_amdgcn_ballot_w64(valid < 32) == 0) {
            switch (width) {
                case 2: encode_round<2, true>(src_row, run, valid, ftab, out, ptr, x); break;
                case 3: encode_round<3, true>(src_row, run, valid, ftab, out, ptr, x); break;
                case 4: encode_round<4, true>(src_row, run, valid, ftab, out, ptr, x); break;
                case 5: encode_round<5, true>(src_row, run, valid, ftab, out, ptr, x); break;
                case 6: encode_round<6, true>(src_row, run, valid, ftab, out, ptr, x); break;
                case 7: encode_round<7, true>(src_row, run, valid, ftab, out, ptr, x); break;
                default: encode_round<8, true>(src_row, run, valid, ftab, out, ptr, x); break;
            }
        } else {
            switch (width) {
                case 2: encode_round<2, false>(src_row, run, valid, ftab, out, ptr, x); break;
                case 3: encode_round<3, false>(src_row, run, valid, ftab, out, ptr, x); break;
                case 4: encode_round<4, false>(src_row, run, valid, ftab, out, ptr, x); break;
                case 5: encode_round<5, false>(src_row, run, valid, ftab, out, ptr, x); break;
                case 6: encode_round<6, false>(src_row, run, valid, ftab, out, ptr, x); break;
                case 7: encode_round<7, false>(src_row, run, valid, ftab, out, ptr, x); break;
                default: encode_round<8, false>(src_row, run, valid, ftab, out, ptr, x); break;
            }
        }
    }
    const uint32_t coders = p.runs < 64u ? p.runs : 64u;  // coders that own a run; the others still hold 2^16
    if (lane < coders) reinterpret_cast<uint32_t *>(slot)[lane] = x;
    if (lane == 0) {
        const uint32_t bytes = 4u * coders + 2u * (cap - ptr);
        len[t] = bytes;                                     // unpadded; the stream is padded to 4 bytes when it is placed
        // padded stream bytes of the token's block of kLenBlock tokens (kLenBlock slots of at most 64 KiB + 256
        // bytes: the sum fits 32 bits)
        atomicAdd(reinterpret_cast<uint32_t *>(ews + e.ws_block) + (t / kLenBlock) * kBlockStride, (bytes + 3u) & ~3u);
    }
}

// A token's stream moves from its slot to its place, by one wave: the (padded) lengths of all streams
// before it are the sums of the blocks before its block plus the lengths before it inside its block
// (64-bit: tokens * slot size may exceed 32 bits; a lane's share stays below 2^40, so it is split at bit
// 24 into two parts whose sums over 64 lanes fit 32 bits).  The first words of the stream are asked for
// together with those lengths: where they come from depends on the token's own length only.  The wave
// of the last token also writes the end offset and the header.
//
// The words stand at the end of the slot's room, which holds an even number of them: they start at an
// odd word exactly when their number is odd.  They move eight at a time (16 bytes; the last ones two at a
// time); in the odd case a pair is the high half of one 32-bit word of the room and the low half of the
// next, and the pair after the last word of the room is the padding to 4 bytes.
struct StreamSource {
    const uint32_t *src;      // the 32-bit word of the room that holds the first word of the stream
    uint32_t left;            // 32-bit words from there to the end of the room
    uint32_t odd;             // the stream starts in the high half of *src
};
__device__ __forceinline__ uint32_t stream_pair(const StreamSource &q, uint32_t i) {
    uint32_t v = q.src[i];
    if (q.odd) v = (v >> 16) | ((i + 1u < q.left ? q.src[i + 1u] : 0u) << 16);
    return v;
}
// pairs 4c .. 4c+3 (all of them exist)
__device__ __forceinline__ Words4 stream_pairs4(const StreamSource &q, uint32_t c) {
    const Words4 a = *reinterpret_cast<const Words4 *>(q.src + 4u * c);
    if (!q.odd) return a;
    const uint32_t next = 4u * c + 4u < q.left ? q.src[4u * c + 4u] : 0u;
    Words4 v;
    v.x = (a.x >> 16) | (a.y << 16); v.y = (a.y >> 16) | (a.z << 16);
    v.z = (a.z >> 16) | (a.w << 16); v.w = (a.w >> 16) | (next << 16);
    return v;
}

constexpr uint32_t kGatherEarly = 2;     // 16-byte pieces per lane that are loaded before the offset is known
__global__ void __launch_bounds__(64)
k_rans_gather(const Params p, const EntropyLayout e, const uint8_t *__restrict__ blob, uint8_t *__restrict__ eblob,
              const uint8_t *__restrict__ ews) {
    static_assert(kLenBlock == 256, "four lengths per lane inside a block");
    if (!blob_is_valid(p, blob)) return;
    const uint32_t t = blockIdx.x, lane = threadIdx.x;
    const uint32_t *len = reinterpret_cast<const uint32_t *>(ews + e.ws_len);
    const uint32_t *block = reinterpret_cast<const uint32_t *>(ews + e.ws_block);
    const uint32_t blk = t / kLenBlock;
    const uint32_t coders = p.runs < 64u ? p.runs : 64u;
    const uint32_t bytes = len[t];                          // states + words, unpadded
    const uint32_t padded = (bytes + 3u) & ~3u;
    const uint32_t room = (e.slot_bytes - 256u) >> 1;
    const uint8_t *slot = ews + e.ws_slots + (size_t)t * e.slot_bytes;
    // (a length that k_rans_encode wrote passes; anything else moves nothing)
    const bool sane = bytes >= 4u * coders && bytes <= e.slot_bytes && ((bytes - 4u * coders) >> 1) <= room;
    const uint32_t nwords = sane ? (bytes - 4u * coders) >> 1 : 0u;
    const uint32_t first = room - nwords, pairs = (nwords + 1u) >> 1, pieces = pairs >> 2;
    StreamSource q;
    q.src = reinterpret_cast<const uint32_t *>(slot + 256) + (first >> 1);
    q.left = (room >> 1) - (first >> 1);
    q.odd = first & 1u;
    Words4 early[kGatherEarly];
#pragma unroll
    for (uint32_t k = 0; k < kGatherEarly; ++k) {
        const uint32_t c = lane + 64u * k;
        early[k] = c < pieces ? stream_pairs4(q, c) : Words4{0u, 0u, 0u, 0u};
    }
    const uint32_t state = lane < coders && sane ? reinterpret_cast<const uint32_t *>(slot)[lane] : 0u;

    uint64_t s = 0;
    for (uint32_t b = lane; b < blk; b += 64u) s += block[b * kBlockStride];
#pragma unroll
    for (uint32_t k = 0; k < kLenBlock / 64u; ++k) {
        const uint32_t u = blk * kLenBlock + lane + 64u * k;
        if (u < t) s += (len[u] + 3u) & ~3u;
    }
    const uint64_t at = (uint64_t)wave_sum_u32((uint32_t)s & 0xFFFFFFu) + ((uint64_t)wave_sum_u32((uint32_t)(s >> 24)) << 24);

    uint64_t *off = reinterpret_cast<uint64_t *>(eblob + e.off_stream_off);
    if (lane == 0) {
        off[t] = at;
        if (t == p.tokens - 1u) {
            off[p.tokens] = at + padded;
            EntropyHeader h = {};
            h.magic = kEntropyMagic; h.version = kVersion; h.tokens = p.tokens; h.hidden = p.hidden;
            h.stream_bytes = at + padded;
            h.off_tables = e.off_tables; h.off_stream_off = e.off_stream_off; h.off_streams = e.off_streams;
            h.stream_capacity = e.stream_capacity;
            *reinterpret_cast<EntropyHeader *>(eblob) = h;
        }
    }
    if (!sane || !stream_move_ok(bytes, coders, e.slot_bytes, at, e.stream_capacity)) return;
    uint8_t *dst = eblob + e.off_streams + at;
    if (lane < coders) reinterpret_cast<uint32_t *>(dst)[lane] = state;
    uint32_t *out = reinterpret_cast<uint32_t *>(dst + 4u * coders);
#pragma unroll
    for (uint32_t k = 0; k < kGatherEarly; ++k) {
        const uint32_t c = lane + 64u * k;
        if (c < pieces) *reinterpret_cast<Words4 *>(out + 4u * c) = early[k];
    }
    for (uint32_t c = lane + 64u * kGatherEarly; c < pieces; c += 64u) *reinterpret_cast<Words4 *>(out + 4u * c) = stream_pairs4(q, c);
    const uint32_t i = 4u * pieces + lane;                  // the last pairs, fewer than four
    if (i < pairs) out[i] = stream_pair(q, i);
}

// ---------------------------------------------------------------- decode

// Inclusive running maximum over the lanes of a wave, in lane order.
__device__ __forceinline__ uint32_t wave_incl_scan_max(uint32_t v) {
    uint32_t n;
    n = dpp<kDppRowShr + 1>(v); v = n > v ? n : v;     // lanes without a source inside their row see 0
    n = dpp<kDppRowShr + 2>(v); v = n > v ? n : v;
    n = dpp<kDppRowShr + 4>(v); v = n > v ? n : v;
    n = dpp<kDppRowShr + 8>(v); v = n > v ? n : v;
    const uint32_t r0 = lane_value(v, 15), r1 = lane_value(v, 31), r2 = lane_value(v, 47);
    const uint32_t row = (threadIdx.x & 63) >> 4;
    uint32_t before = 0;
    if (row > 0) before = r0;
    if (row > 1) before = r1 > before ? r1 : before;
    if (row > 2) before = r2 > before ? r2 : before;
    return v > before ? v : before;
}

// slot -> code for all 4096 slots: a code's index is written at the slot where its range starts,
// and a running maximum carries it over the range (later codes start at later slots).
__device__ __forceinline__ void build_slot_table(const uint32_t *ftab, uint32_t *sym32) {
    const uint32_t lane = threadIdx.x & 63u;
    uint8_t *sym = reinterpret_cast<uint8_t *>(sym32);
#pragma unroll
    for (int i = 0; i < 16; ++i) sym32[16u * lane + i] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t c = 4u * lane + i, fc = ftab[c];
        if (fc & 0xFFFFu) sym[frequency_slot(fc >> 16)] = (uint8_t)c;   // masked: a damaged table stays inside the array
    }
    __syncthreads();
    // lane l owns the slots 64l .. 64l+63
    uint32_t w[16], mx = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        w[i] = sym32[16u * lane + i];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t v = (w[i] >> (8 * k)) & 0xFFu;
            mx = v > mx ? v : mx;
        }
    }
    const uint32_t incl = wave_incl_scan_max(mx);
    // the maximum over the lanes before this one: shift the inclusive result down by one lane
    uint32_t run = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((lane + 63u) & 63u) << 2), (int)incl);
    if (lane == 0) run = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        uint32_t o = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t v = (w[i] >> (8 * k)) & 0xFFu;
            run = v > run ? v : run;
            o |= run << (8 * k);
        }
        sym32[16u * lane + i] = o;
    }
    __syncthreads();
}

// The token's words as the decoder consumes them: windows of 64 words in registers (lane l of window k
// holds word base + 64k + l).  A step reads at most 64 words from the first two windows, which share a
// register (low / high half: one permute reads both); when the first is used up the windows move on by
// one.  Behind them: two registers of two windows each (pair, next) and two of one window each (far),
// which move on by two windows at every second move, when two new windows are asked for.  So a window is
// not touched until two moves after it was asked for: by then it has arrived (a window is a cache line of
// its own, fetched from memory for the first time), and no step waits for memory.
// Past the end of the stream a window repeats the stream's last word: a stream that is not damaged is never
// read there.
struct Words {
    const uint16_t *src;
    uint32_t last, base;       // index of the last word; first word of the first window
    uint32_t cur;              // the first two windows
    uint32_t pair, next;       // windows 0, 1 and 2, 3 (odd = 0) or -1, 0 and 1, 2 (odd = 1)
    uint32_t far0, far1;       // the two windows after those
    uint32_t odd;              // one window of `pair` is used up
};
__device__ __forceinline__ uint32_t word_at(const Words &q, uint32_t k) {
    const uint32_t i = k + (threadIdx.x & 63u);
    return (uint32_t)q.src[i < q.last ? i : q.last];
}
// count words at src; `fallback` is readable memory for the case of no words at all
__device__ __forceinline__ void words_open(Words &q, const uint16_t *src, uint32_t count, const uint16_t *fallback) {
    q.src = count ? src : fallback; q.last = count ? count - 1u : 0u; q.base = 0; q.odd = 0;
    q.pair = word_at(q, 0) | (word_at(q, 64) << 16); q.next = word_at(q, 128) | (word_at(q, 192) << 16);
    q.far0 = word_at(q, 256); q.far1 = word_at(q, 320);
    q.cur = q.pair;
}
// the first window is used up
__device__ __forceinline__ void words_move_on(Words &q) {
    q.base += 64u;
    if (q.odd) {                                              // (uniform)
        q.pair = q.next;
        q.next = q.far0 | (q.far1 << 16);
        // (the loads stay behind the last use of the registers they fill: moved ahead of it, they would need
        // other registers and copies, which would wait for them)
        asm volatile("; the far windows have moved, their registers are asked for again" : "+v"(q.pair), "+v"(q.next) : : "memory");
        q.far0 = word_at(q, q.base + 256u);
        q.far1 = word_at(q, q.base + 320u);
    }
    q.odd ^= 1u;
    q.cur = q.odd ? (q.pair >> 16) | (q.next << 16) : q.pair;
}

// A SIMD holds the waves of eight tokens, each a chain of dependent steps, and its arbiter prefers the oldest
// wave: left alone, the waves finish one after the other and the last ones run with the SIMD half idle.  A wave
// therefore lowers its issue priority as it gets ahead (by quarters of its rounds), which keeps the eight in
// step: the decoder of C4 takes 54 us instead of 60.  (The encoder, whose steps wait less, gains nothing from it.)
// `done` of `total` rounds are behind the wave (uniform).
__device__ __forceinline__ void priority_by_progress(uint32_t done, uint32_t total) {
    switch ((4u * done) / total) {
        case 0: __builtin_amdgcn_s_setprio(3); break;
        case 1: __builtin_amdgcn_s_setprio(2); break;
        case 2: __builtin_amdgcn_s_setprio(1); break;
        default: __builtin_amdgcn_s_setprio(0); break;
    }
}

template <int B, bool WHOLE>
__device__ __forceinline__ void decode_round(uint32_t *dst_row, uint32_t run, int valid, const uint32_t *ftab,
                                             const uint8_t *sym, Words &q, uint32_t &pos, uint32_t &x) {
    uint32_t d[B];
#pragma unroll
    for (int k = 0; k < B; ++k) d[k] = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const bool active = WHOLE || j < valid;
        const uint32_t slot = frequency_slot(x);
        const uint32_t s = sym[slot];
        const uint32_t fc = ftab[s];
        if (active) {
            x = __umul24(fc & 0xFFFFu, x >> kProbBits) + slot - (fc >> 16);    // f <= 2^12, x >> 12 < 2^20
            const int off = j * B, k = off >> 5, sh = off & 31;
            d[k] |= s << sh;
            if (sh + B > 32) d[k + 1 < B ? k + 1 : k] |= s >> (32 - sh);
        }
        const bool need = active && x < kRansLow;
        const uint64_t who = __builtin_amdgcn_ballot_w64(need);
        if (who) {
            const uint32_t at = pos - q.base + rank_in(who);   // < 128
            const uint32_t both = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((at & 63u) << 2), (int)q.cur);
            if (need) x = (x << 16) | ((both >> ((at & 64u) >> 2)) & 0xFFFFu);
            pos += (uint32_t)__builtin_popcountll(who);
            if (pos - q.base >= 64u) words_move_on(q);
        }
    }
    const uint32_t nd = (WHOLE || valid >= 32) ? (uint32_t)B : (valid > 0 ? ((uint32_t)valid * B + 31u) >> 5 : 0u);
    if (WHOLE) {
        store_run_words<B>(dst_row + run * B, d);
    } else {
#pragma unroll
        for (int k = 0; k < B; ++k)
            if ((uint32_t)k < nd) dst_row[run * B + k] = d[k];
    }
}

__global__ void __launch_bounds__(64, 8)    // 8 waves per SIMD: all 32 tokens of a compute unit's share run at once
k_rans_decode(const Params p, const EntropyLayout e, const uint8_t *__restrict__ eblob, uint8_t *__restrict__ blob) {
    __shared__ uint32_t ftab[256];
    __shared__ uint32_t sym32[1024];                                   // slot -> code, one byte per slot
    const uint32_t t = blockIdx.x, lane = threadIdx.x;
    if (!blob_is_valid(p, blob) || !eblob_is_valid(p, e, eblob)) return;
    const uint32_t width = blob[p.off_bits + t];
    const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
    if (!token_in_range(p, width, po)) return;
    const uint64_t *off = reinterpret_cast<const uint64_t *>(eblob + e.off_stream_off);
    const uint64_t a = off[t], b = off[t + 1];
    const uint32_t coders = p.runs < 64u ? p.runs : 64u;  // states in the stream; the other coders start (and stay) at 2^16
    if (!stream_span_ok(a, b, e.stream_capacity, coders, e.slot_bytes)) return;
    load_table_decode(reinterpret_cast<const uint16_t *>(eblob + e.off_tables) + (width - 2u) * 256u, ftab);
    __syncthreads();
    build_slot_table(ftab, sym32);
    const uint8_t *sym = reinterpret_cast<const uint8_t *>(sym32);
    const uint8_t *stream = eblob + e.off_streams + a;
    Words q;
    words_open(q, reinterpret_cast<const uint16_t *>(stream + 4u * coders), (uint32_t)(b - a - 4u * coders) >> 1,
               reinterpret_cast<const uint16_t *>(stream));
    uint32_t x = lane < coders ? reinterpret_cast<const uint32_t *>(stream)[lane] : kRansLow, pos = 0;
    uint32_t *dst_row = reinterpret_cast<uint32_t *>(blob + p.off_payload + po);
    const uint32_t rounds = (p.runs + 63u) / 64u;
    for (uint32_t r = 0; r < rounds; ++r) {
        priority_by_progress(r, rounds);
        const uint32_t run = lane + 64u * r;
        const int valid = (int)p.hidden - (int)(run * kRun);
        if (__builtin_amdgcn_ballot_w64(valid < 32) == 0) {
            switch (width) {
                case 2: decode_round<2, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 3: decode_round<3, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 4: decode_round<4, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 5: decode_round<5, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 6: decode_round<6, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 7: decode_round<7, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                default: decode_round<8, true>(dst_row, run, valid, ftab, sym, q, pos, x); break;
            }
        } else {
            switch (width) {
                case 2: decode_round<2, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 3: decode_round<3, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 4: decode_round<4, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 5: decode_round<5, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 6: decode_round<6, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                case 7: decode_round<7, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
                default: decode_round<8, false>(dst_row, run, valid, ftab, sym, q, pos, x); break;
            }
        }
    }
}

// ---------------------------------------------------------------- launchers

static hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

int launch_rans_encode(const Params &p, const Geometry &g, const EntropyLayout &e, const void *d_blob, void *d_eblob,
                       void *d_ews, void *stream) {
    const uint8_t *blob = static_cast<const uint8_t *>(d_blob);
    uint8_t *eblob = static_cast<uint8_t *>(d_eblob), *ews = static_cast<uint8_t *>(d_ews);
    hipStream_t s = as_stream(stream);
    const uint32_t to_zero = kPoolCopies * 7u * 256u + (p.tokens + kLenBlock - 1u) / kLenBlock;
    hipLaunchKernelGGL(k_rans_begin, dim3((to_zero + kBeginThreads - 1u) / kBeginThreads), dim3(kBeginThreads), 0, s, p, e, eblob, ews);
    int rc = launch_code_pool(p, g, e, d_blob, ews + e.ws_pooled, stream);
    if (rc != 0) return rc;
    hipLaunchKernelGGL(k_rans_tables, dim3(7), dim3(256), 0, s, p, e, blob, eblob, ews);
    hipLaunchKernelGGL(k_rans_encode, dim3(p.tokens), dim3(64), 0, s, p, e, blob, eblob, ews);
    hipLaunchKernelGGL(k_rans_gather, dim3(p.tokens), dim3(64), 0, s, p, e, blob, eblob, ews);
    return (int)hipGetLastError();
}

int launch_rans_decode(const Params &p, const EntropyLayout &e, const void *d_eblob, void *d_blob, void *stream) {
    hipLaunchKernelGGL(k_rans_decode, dim3(p.tokens), dim3(64), 0, as_stream(stream), p, e,
                       static_cast<const uint8_t *>(d_eblob), static_cast<uint8_t *>(d_blob));
    return (int)hipGetLastError();
}

}  // namespace tsq
