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
// (k_rans_encode) -> stream bytes per block of 256 tokens (k_rans_blocks) -> every token finds its
// offset from the block sums before it and the lengths before it inside its block, and its stream
// moves to its place (k_rans_gather).
// Decode: one wave per token (k_rans_decode) rebuilds the packed payload; the words it reads
// pass through registers (four windows of 64 words), so a token needs 5 KB of LDS for its tables
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

__global__ void k_rans_begin(const Params p, const EntropyLayout e, uint8_t *__restrict__ eblob, uint8_t *__restrict__ ews) {
    uint32_t *counts = reinterpret_cast<uint32_t *>(ews + e.ws_pooled);
    for (uint32_t i = threadIdx.x; i < kPoolCopies * 7u * 256u; i += blockDim.x) counts[i] = 0;
    // the header becomes valid only when the last kernel of the call has run
    if (threadIdx.x < sizeof(EntropyHeader) / 4) reinterpret_cast<uint32_t *>(eblob)[threadIdx.x] = 0;
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
// x = f | cum << 16 (cum = exclusive running sum, < 4096) and y = the binary32 pattern of 1 / f.
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
        ftab[4u * lane + i] = make_uint2(fi | (cum << 16), __float_as_uint(1.0f / (float)fi));
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

// x / f and x % f for x < f << 20 (so the quotient is below 2^20) and f <= 4096: the binary32
// product of x and 1/f is within 0.2 of the true quotient (three roundings of relative size
// 2^-24 on a value below 2^20), so its integer part is off by at most one, which the sign and
// size of the remainder tell.  All multiplications fit 24 bits.
__device__ __forceinline__ void divide_small(uint32_t x, uint32_t f, float rcp, uint32_t &q, uint32_t &r) {
    uint32_t qq = (uint32_t)((float)x * rcp);
    int32_t rr = (int32_t)(x - __umul24(qq, f));
    if (rr < 0) { --qq; rr += (int32_t)f; }
    else if ((uint32_t)rr >= f) { ++qq; rr -= (int32_t)f; }
    q = qq;
    r = (uint32_t)rr;
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
#pragma unroll
    for (int k = 0; k < B; ++k) d[k] = (WHOLE || (uint32_t)k < nd) ? src_row[run * B + k] : 0u;
#pragma unroll
    for (int j = 31; j >= 0; --j) {
        const int off = j * B, k = off >> 5, sh = off & 31;
        uint32_t code = d[k] >> sh;
        if (sh + B > 32) code |= d[k + 1 < B ? k + 1 : k] << (32 - sh);
        code &= (1u << B) - 1u;
        const bool active = WHOLE || j < valid;
        const uint2 entry = ftab[code];
        const uint32_t f = entry.x & 0xFFFFu;
        const uint32_t c = entry.x >> 16;
        const bool shed = active && (x >> 20) >= f;            // x >= f << 20, without overflow for f = 4096
        const uint64_t who = __builtin_amdgcn_ballot_w64(shed);
        ptr -= (uint32_t)__builtin_popcountll(who);
        if (shed) {
            out[ptr + rank_in(who)] = (uint16_t)x;
            x >>= 16;
        }
        if (active) {
            uint32_t q, r;
            divide_small(x, f, __uint_as_float(entry.y), q, r);
            x = (q << kProbBits) + r + c;
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
        len[t] = 4u * coders + 2u * (cap - ptr);           // unpadded; the stream is padded to 4 bytes when it is placed
    }
}

// Padded stream bytes of every block of kLenBlock tokens: one workgroup per block, one thread per
// token.  kLenBlock slots of at most 64 KiB + 256 bytes: the sum fits 32 bits.
__global__ void __launch_bounds__(256)
k_rans_blocks(const Params p, const EntropyLayout e, const uint8_t *__restrict__ blob, uint8_t *__restrict__ ews) {
    __shared__ uint32_t part[4];
    static_assert(kLenBlock == 256, "one thread per token of a block");
    if (!blob_is_valid(p, blob)) return;
    const uint32_t *len = reinterpret_cast<const uint32_t *>(ews + e.ws_len);
    const uint32_t t = blockIdx.x * kLenBlock + threadIdx.x;
    const uint32_t w = wave_sum_u32(t < p.tokens ? (len[t] + 3u) & ~3u : 0u);
    if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) reinterpret_cast<uint32_t *>(ews + e.ws_block)[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// A token's stream moves from its slot to its place: the (padded) lengths of all streams before it
// are the sums of the blocks before its block plus the lengths before it inside its block, added up
// by the workgroup (64-bit: tokens * slot size may exceed 32 bits; a thread's share stays below
// 2^34, so it is split at bit 24 into two parts whose sums over 256 threads fit 32 bits).  The
// workgroup of the last token also writes the end offset and the header.
__global__ void __launch_bounds__(256)
k_rans_gather(const Params p, const EntropyLayout e, const uint8_t *__restrict__ blob, uint8_t *__restrict__ eblob,
              const uint8_t *__restrict__ ews) {
    __shared__ uint32_t part[2][4];
    static_assert(kLenBlock == 256, "one thread per token of a block");
    if (!blob_is_valid(p, blob)) return;
    const uint32_t t = blockIdx.x;
    const uint32_t *len = reinterpret_cast<const uint32_t *>(ews + e.ws_len);
    const uint32_t *block = reinterpret_cast<const uint32_t *>(ews + e.ws_block);
    const uint32_t blk = t / kLenBlock;
    uint64_t s = 0;
    for (uint32_t b = threadIdx.x; b < blk; b += 256u) s += block[b];
    const uint32_t u = blk * kLenBlock + threadIdx.x;       // kLenBlock == threads of this workgroup
    if (u < t) s += (len[u] + 3u) & ~3u;
    const uint32_t lo = wave_sum_u32((uint32_t)s & 0xFFFFFFu), hi = wave_sum_u32((uint32_t)(s >> 24));
    if ((threadIdx.x & 63u) == 0) { part[0][threadIdx.x >> 6] = lo; part[1][threadIdx.x >> 6] = hi; }
    __syncthreads();
    uint64_t at = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) at += (uint64_t)part[0][w] + ((uint64_t)part[1][w] << 24);

    const uint32_t bytes = len[t];                          // states + words, unpadded
    const uint32_t padded = (bytes + 3u) & ~3u;
    uint64_t *off = reinterpret_cast<uint64_t *>(eblob + e.off_stream_off);
    if (threadIdx.x == 0) {
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
    const uint32_t coders = p.runs < 64u ? p.runs : 64u;
    if (!stream_move_ok(bytes, coders, e.slot_bytes, at, e.stream_capacity)) return;
    const uint8_t *slot = ews + e.ws_slots + (size_t)t * e.slot_bytes;
    uint8_t *dst = eblob + e.off_streams + at;
    if (threadIdx.x < coders) reinterpret_cast<uint32_t *>(dst)[threadIdx.x] = reinterpret_cast<const uint32_t *>(slot)[threadIdx.x];
    // the words stand at the end of the slot
    const uint32_t nwords = (bytes - 4u * coders) >> 1, room = (e.slot_bytes - 256u) >> 1;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(slot + 256) + (room - nwords);
    uint16_t *words = reinterpret_cast<uint16_t *>(dst + 4u * coders);
    for (uint32_t i = threadIdx.x; i < nwords; i += 256u) words[i] = src[i];
    if ((nwords & 1u) && threadIdx.x == 0) words[nwords] = 0;                          // padding to 4 bytes
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

// The token's words as the decoder consumes them: four windows of 64 words in registers (lane l
// of window k holds word base + 64k + l); a step reads at most 64 words from the first two, and
// when the first is used up the windows move on and the fourth is fetched from memory again.
struct Words {
    const uint16_t *src;
    uint32_t count, base;
    uint32_t w01, w2, w3;      // the first two windows share a register (low / high half): one permute reads both
};
__device__ __forceinline__ uint32_t word_at(const Words &q, uint32_t k) {
    const uint32_t i = k + (threadIdx.x & 63u);
    return i < q.count ? (uint32_t)q.src[i] : 0u;               // past the end: a damaged stream is read as zeros
}
__device__ __forceinline__ void words_open(Words &q, const uint16_t *src, uint32_t count) {
    q.src = src; q.count = count; q.base = 0;
    q.w01 = word_at(q, 0) | (word_at(q, 64) << 16); q.w2 = word_at(q, 128); q.w3 = word_at(q, 192);
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
            const uint32_t both = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((at & 63u) << 2), (int)q.w01);
            if (need) x = (x << 16) | ((both >> ((at & 64u) >> 2)) & 0xFFFFu);
            pos += (uint32_t)__builtin_popcountll(who);
            if (pos - q.base >= 64u) {
                q.base += 64u;
                q.w01 = (q.w01 >> 16) | (q.w2 << 16); q.w2 = q.w3;
                q.w3 = word_at(q, q.base + 192u);
            }
        }
    }
    const uint32_t nd = (WHOLE || valid >= 32) ? (uint32_t)B : (valid > 0 ? ((uint32_t)valid * B + 31u) >> 5 : 0u);
#pragma unroll
    for (int k = 0; k < B; ++k)
        if (WHOLE || (uint32_t)k < nd) dst_row[run * B + k] = d[k];
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
    words_open(q, reinterpret_cast<const uint16_t *>(stream + 4u * coders), (uint32_t)(b - a - 4u * coders) >> 1);
    uint32_t x = lane < coders ? reinterpret_cast<const uint32_t *>(stream)[lane] : kRansLow, pos = 0;
    uint32_t *dst_row = reinterpret_cast<uint32_t *>(blob + p.off_payload + po);
    const uint32_t rounds = (p.runs + 63u) / 64u;
    for (uint32_t r = 0; r < rounds; ++r) {
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
    hipLaunchKernelGGL(k_rans_begin, dim3(1), dim3(1024), 0, s, p, e, eblob, ews);
    int rc = launch_code_pool(p, g, e, d_blob, ews + e.ws_pooled, stream);
    if (rc != 0) return rc;
    hipLaunchKernelGGL(k_rans_tables, dim3(7), dim3(256), 0, s, p, e, blob, eblob, ews);
    hipLaunchKernelGGL(k_rans_encode, dim3(p.tokens), dim3(64), 0, s, p, e, blob, eblob, ews);
    hipLaunchKernelGGL(k_rans_blocks, dim3((p.tokens + kLenBlock - 1u) / kLenBlock), dim3(256), 0, s, p, e, blob, ews);
    hipLaunchKernelGGL(k_rans_gather, dim3(p.tokens), dim3(256), 0, s, p, e, blob, eblob, ews);
    return (int)hipGetLastError();
}

int launch_rans_decode(const Params &p, const EntropyLayout &e, const void *d_eblob, void *d_blob, void *stream) {
    hipLaunchKernelGGL(k_rans_decode, dim3(p.tokens), dim3(64), 0, as_stream(stream), p, e,
                       static_cast<const uint8_t *>(d_eblob), static_cast<uint8_t *>(d_blob));
    return (int)hipGetLastError();
}

}  // namespace tsq
