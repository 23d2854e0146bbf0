// Symbol statistics of a compressed blob (gfx950): the first stage of the entropy coder that the
// paper places after TAB-Q (Sec. II-C.2, last paragraph: the quantized symbols go to an rANS
// coder).  An adaptive coder needs, per token, how often each of the 2^b_t codes occurs.
//
// Counting happens in LDS with atomic adds on several interleaved copies of the bins (a lane uses
// the copy lane % copies), which keeps the few frequent codes of a narrow width from meeting in one
// word; the copies are added up at the end.  A run of 32 codes is read with as few memory instructions
// as its width allows.
#include <hip/hip_runtime.h>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

constexpr uint32_t kCountAhead = 4;      // runs of a lane that are loaded before the first of them is counted

// A token per wave (the pooled counts): lane l takes the runs l, l + 64, ... of 32 codes, as the coder
// does, four runs on their way at a time.  The count of code c goes to mine[c * COPIES]; what lies
// beyond the end of the row is not counted.
template <int B, uint32_t COPIES>
__device__ __forceinline__ void count_token(const Params &p, const uint32_t *row, uint32_t rounds, uint32_t *mine) {
    const uint32_t lane = threadIdx.x & 63u;
    for (uint32_t r0 = 0; r0 < rounds; r0 += kCountAhead) {
        uint32_t d[kCountAhead][B], valid[kCountAhead];
#pragma unroll
        for (uint32_t k = 0; k < kCountAhead; ++k) {
            const uint32_t run = lane + 64u * (r0 + k), first = run * kRun;
            valid[k] = first < p.hidden ? (p.hidden - first < 32u ? p.hidden - first : 32u) : 0u;
            if (valid[k] == 32u) {
                load_run_words<B>(row + run * B, d[k]);
            } else {
                const uint32_t nd = (valid[k] * B + 31u) >> 5;
#pragma unroll
                for (uint32_t w = 0; w < (uint32_t)B; ++w) d[k][w] = w < nd ? row[run * B + w] : 0u;
            }
        }
#pragma unroll
        for (uint32_t k = 0; k < kCountAhead; ++k) {
            if (r0 + k >= rounds) break;                       // (its lanes loaded nothing: their runs lie beyond the row)
            const bool ragged = __builtin_amdgcn_ballot_w64(valid[k] < 32u) != 0;
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int off = j * B, w = off >> 5, sh = off & 31;
                uint32_t code = d[k][w] >> sh;
                if (sh + B > 32) code |= d[k][w + 1 < B ? w + 1 : w] << (32 - sh);
                code &= (1u << B) - 1u;
                if (!ragged || (uint32_t)j < valid[k])
                    __hip_atomic_fetch_add(mine + code * COPIES, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
}
template <uint32_t COPIES>
__device__ __forceinline__ void count_token_any(const Params &p, uint32_t b, const uint32_t *row, uint32_t rounds,
                                                uint32_t *mine) {
    switch (b) {                                               // uniform in the wave
        case 2: count_token<2, COPIES>(p, row, rounds, mine); break;
        case 3: count_token<3, COPIES>(p, row, rounds, mine); break;
        case 4: count_token<4, COPIES>(p, row, rounds, mine); break;
        case 5: count_token<5, COPIES>(p, row, rounds, mine); break;
        case 6: count_token<6, COPIES>(p, row, rounds, mine); break;
        case 7: count_token<7, COPIES>(p, row, rounds, mine); break;
        default: count_token<8, COPIES>(p, row, rounds, mine); break;
    }
}

__device__ __forceinline__ bool blob_is_this_plans(const Params &p, const uint8_t *blob) {
    const BlobHeader *h = reinterpret_cast<const BlobHeader *>(blob);
    return h->magic == kMagic && h->version == kVersion && h->status == 0 && h->tokens == p.tokens &&
           h->hidden == p.hidden && h->dtype == p.dtype && h->off_payload == p.off_payload;
}

// Per token: hist[t][c] = how often code c occurs in token t.  One workgroup per token, one lane per run of
// 32 codes, as in k_unpack; kCopies copies of the 256 bins, 257 words apart (equal codes of different
// copies fall into different banks), added up at the end, one bin per thread.  (A wave per token with
// bins of its own would need no barriers, but has room for four copies only, and with four the atomic
// adds of equal codes meet in one word so often that it is slower.)
constexpr uint32_t kCopies = 16, kCopyStride = 257;

// The 32 codes of a run into the lane's copy of the bins.  RAGGED: the run may reach past the end
// of the row; what lies beyond is counted in the copy's spare word (index 256) instead of being
// branched around.
template <int B, bool RAGGED>
__device__ __forceinline__ void count_run(const uint32_t *src_row, uint32_t run, uint32_t valid_elems, uint32_t *bins) {
    uint32_t d[B];
    const uint32_t *src = src_row + run * B;
    const uint32_t nd = (!RAGGED || valid_elems >= 32u) ? (uint32_t)B : (valid_elems * B + 31u) >> 5;
    if (!RAGGED) {
        load_run_words<B>(src, d);
    } else {
#pragma unroll
        for (int k = 0; k < B; ++k) d[k] = (uint32_t)k < nd ? src[k] : 0u;
    }
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const int off = j * B, k = off >> 5, sh = off & 31;
        uint32_t code = d[k] >> sh;
        if (sh + B > 32) code |= d[k + 1 < B ? k + 1 : k] << (32 - sh);
        code &= (1u << B) - 1u;
        if (RAGGED && (uint32_t)j >= valid_elems) code = 256u;
        __hip_atomic_fetch_add(bins + code, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}
template <bool RAGGED>
__device__ __forceinline__ void count_run_any(uint32_t width, const uint32_t *src_row, uint32_t run, uint32_t valid_elems,
                                              uint32_t *bins) {
    switch (width) {
        case 2: count_run<2, RAGGED>(src_row, run, valid_elems, bins); break;
        case 3: count_run<3, RAGGED>(src_row, run, valid_elems, bins); break;
        case 4: count_run<4, RAGGED>(src_row, run, valid_elems, bins); break;
        case 5: count_run<5, RAGGED>(src_row, run, valid_elems, bins); break;
        case 6: count_run<6, RAGGED>(src_row, run, valid_elems, bins); break;
        case 7: count_run<7, RAGGED>(src_row, run, valid_elems, bins); break;
        default: count_run<8, RAGGED>(src_row, run, valid_elems, bins); break;
    }
}

__global__ void __launch_bounds__(1024)
k_code_hist(const Params p, const uint8_t *__restrict__ blob, uint32_t *__restrict__ hist) {
    __shared__ uint32_t bins[kCopies * kCopyStride];
    const uint32_t t = blockIdx.x, run = threadIdx.x;

    // the blob must be this plan's and must have been completed without error
    const BlobHeader *h = reinterpret_cast<const BlobHeader *>(blob);
    if (h->magic != kMagic || h->version != kVersion || h->status != 0 || h->tokens != p.tokens ||
        h->hidden != p.hidden || h->dtype != p.dtype || h->off_payload != p.off_payload)
        return;
    const uint32_t width = blob[p.off_bits + t];
    const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
    // a damaged token is skipped rather than read out of bounds
    if (!token_in_range(p, width, po)) return;

    for (uint32_t i = threadIdx.x; i < kCopies * kCopyStride; i += blockDim.x) bins[i] = 0;
    __syncthreads();
    if (run < p.runs) {
        const uint32_t left = p.hidden - run * kRun;
        const uint32_t *src_row = reinterpret_cast<const uint32_t *>(blob + p.off_payload + po);
        uint32_t *mine = bins + (threadIdx.x & (kCopies - 1u)) * kCopyStride;
        // whole runs everywhere in this wave (always, unless the row ends inside it): no range checks
        if (__builtin_amdgcn_ballot_w64(left < 32u) == 0) count_run_any<false>(width, src_row, run, left, mine);
        else count_run_any<true>(width, src_row, run, left, mine);
    }
    __syncthreads();
    for (uint32_t c = threadIdx.x; c < 256u; c += blockDim.x) {
        uint32_t n = 0;
#pragma unroll
        for (uint32_t k = 0; k < kCopies; ++k) n += bins[k * kCopyStride + c];
        hist[(size_t)t * 256u + c] = n;
    }
}

// The same counts pooled per width class (what the frequency tables of the entropy coder are built
// from).  A workgroup of sixteen waves counts `per` consecutive tokens into bins that stay in LDS until
// all its tokens are counted: one bin per (width, code) pair and lane % 16, word
// (2^b - 4 + code) * 16 + lane % 16; that is 508 pairs.  At the end thread k adds up the 16 words of
// pair k and adds the sum to one of kPoolCopies sets counts[set][7][256] (row b - 2: width b; zeroed
// by the caller), which k_rans_tables adds up: atomic adds on one address from all over the chip
// take about 30 ns each, one after the other, so both the number of counting workgroups and the
// number of them that share a set are kept small.
constexpr uint32_t kPoolPairs = 508, kPoolLanes = 16, kPoolWords = kPoolPairs * kPoolLanes;
constexpr uint32_t kPoolThreads = 1024, kPoolWaves = kPoolThreads / 64;
__global__ void __launch_bounds__(kPoolThreads, 8)     // 8 waves per SIMD (two workgroups per compute unit): at most 64 vector registers
k_code_pool(const Params p, const uint8_t *__restrict__ blob, uint32_t *__restrict__ counts, uint32_t per) {
    __shared__ uint32_t bins[kPoolWords];
    if (!blob_is_this_plans(p, blob)) return;
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
    const uint32_t t0 = blockIdx.x * per, t1 = t0 + per < p.tokens ? t0 + per : p.tokens;
    const uint32_t rounds = (p.runs + 63u) / 64u;
    // width and place of the wave's first token are on their way while the bins are cleared
    uint32_t t = uniform(t0 + wv);
    uint32_t b_next = t < t1 ? blob[p.off_bits + t] : 0u;
    uint64_t po_next = t < t1 ? reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t] : 0u;
    for (uint32_t i = threadIdx.x; i < kPoolWords; i += kPoolThreads) bins[i] = 0;
    __syncthreads();

    uint32_t *mine = bins + (lane & (kPoolLanes - 1u));
    for (; t < t1; t += kPoolWaves) {
        // (the same in every lane: kept in scalar registers)
        const uint32_t b = uniform(b_next);
        const uint64_t po = (uint64_t)uniform((uint32_t)po_next) | ((uint64_t)uniform((uint32_t)(po_next >> 32)) << 32);
        if (t + kPoolWaves < t1) {
            b_next = blob[p.off_bits + t + kPoolWaves];
            po_next = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t + kPoolWaves];
        }
        if (!token_in_range(p, b, po)) continue;               // a damaged token is skipped rather than read out of bounds
        const uint32_t *row = reinterpret_cast<const uint32_t *>(blob + p.off_payload + po);
        count_token_any<kPoolLanes>(p, b, row, rounds, mine + ((1u << b) - 4u) * kPoolLanes);
    }
    __syncthreads();
    if (threadIdx.x < kPoolPairs) {
        const uint32_t pair = threadIdx.x;
        uint32_t n = 0;
#pragma unroll
        for (uint32_t k = 0; k < kPoolLanes; ++k) n += bins[pair * kPoolLanes + ((k + pair) & (kPoolLanes - 1u))];
        // pair = 2^b - 4 + code
        const uint32_t bw = 31u - (uint32_t)__builtin_clz(pair + 4u), code = pair + 4u - (1u << bw);
        if (n) atomicAdd(counts + (blockIdx.x % kPoolCopies) * 7u * 256u + (bw - 2u) * 256u + code, n);
    }
}

int launch_code_hist(const Params &p, const Geometry &g, const void *d_blob, void *d_hist, void *stream) {
    hipLaunchKernelGGL(k_code_hist, dim3(p.tokens), dim3(g.block), 0, reinterpret_cast<hipStream_t>(stream), p,
                       static_cast<const uint8_t *>(d_blob), static_cast<uint32_t *>(d_hist));
    return (int)hipGetLastError();
}

int launch_code_pool(const Params &p, const Geometry &g, const EntropyLayout &e, const void *d_blob, void *d_counts,
                     void *stream) {
    hipLaunchKernelGGL(k_code_pool, dim3(e.pool_groups), dim3(kPoolThreads), 0, reinterpret_cast<hipStream_t>(stream), p,
                       static_cast<const uint8_t *>(d_blob), static_cast<uint32_t *>(d_counts), e.pool_tokens);
    return (int)hipGetLastError();
}

}  // namespace tsq
