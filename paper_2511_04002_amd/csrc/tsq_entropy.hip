// Symbol statistics of a compressed blob (gfx950): the first stage of the entropy coder that the
// paper places after TAB-Q (Sec. II-C.2, last paragraph: the quantized symbols go to an rANS
// coder).  An adaptive coder needs, per token, how often each of the 2^b_t codes occurs.
//
// One workgroup per token, one lane per run of 32 codes, as in k_unpack.  Counting happens in
// LDS with atomic adds on kCopies interleaved copies of the 256 bins (a lane uses the copy
// lane % kCopies; copies are 257 words apart so that equal codes of different copies fall into
// different banks), which keeps the few frequent codes of a narrow width from serializing the
// whole wave on one address.  The copies are added up at the end, one bin per thread.
#include <hip/hip_runtime.h>

#include "tsq_device.hpp"
#include "tsq_internal.hpp"

namespace tsq {

constexpr uint32_t kCopies = 16, kCopyStride = 257;

// The 32 codes of a run into the lane's copy of the bins.  RAGGED: the run may reach past the end
// of the row; what lies beyond is counted in the copy's spare word (index 256) instead of being
// branched around.
template <int B, bool RAGGED>
__device__ __forceinline__ void count_run(const uint32_t *src_row, uint32_t run, uint32_t valid_elems, uint32_t *bins) {
    uint32_t d[B];
    const uint32_t *src = src_row + run * B;
    const uint32_t nd = (!RAGGED || valid_elems >= 32u) ? (uint32_t)B : (valid_elems * B + 31u) >> 5;
#pragma unroll
    for (int k = 0; k < B; ++k) d[k] = (!RAGGED || (uint32_t)k < nd) ? src[k] : 0u;
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
// from).  A workgroup counts `per` consecutive tokens, class by class: all its tokens of one width
// go into the bins before the copies are added up, so the adding up happens once per width that
// occurs, not once per token.  The sums are added to one of kPoolCopies sets counts[set][7][256]
// (row b - 2: width b; zeroed by the caller), which k_rans_tables adds up: atomic adds on one
// address from all over the chip take about 30 ns each, one after the other, so both the number
// of counting workgroups and the number of them that share a set are kept small.
constexpr uint32_t kPoolMaxTokens = 64;   // widths held in LDS at a time
__global__ void __launch_bounds__(1024)
k_code_pool(const Params p, const uint8_t *__restrict__ blob, uint32_t *__restrict__ counts, uint32_t per) {
    __shared__ uint32_t bins[kCopies * kCopyStride];
    __shared__ uint32_t acc[7 * 256];
    __shared__ uint8_t widths[kPoolMaxTokens];
    const BlobHeader *h = reinterpret_cast<const BlobHeader *>(blob);
    const bool ok = h->magic == kMagic && h->version == kVersion && h->status == 0 && h->tokens == p.tokens &&
                    h->hidden == p.hidden && h->dtype == p.dtype && h->off_payload == p.off_payload;
    const uint32_t run = threadIdx.x;
    uint32_t *mine_out = counts + (blockIdx.x % kPoolCopies) * 7u * 256u;
    for (uint32_t i = threadIdx.x; i < 7u * 256u; i += blockDim.x) acc[i] = 0;
    for (uint32_t i = threadIdx.x; i < kCopies * kCopyStride; i += blockDim.x) bins[i] = 0;
    const uint32_t t0 = blockIdx.x * per, t1 = t0 + per < p.tokens ? t0 + per : p.tokens;
    for (uint32_t base = t0; ok && base < t1; base += kPoolMaxTokens) {
        const uint32_t n = t1 - base < kPoolMaxTokens ? t1 - base : kPoolMaxTokens;
        __syncthreads();                                   // bins and acc are zero / complete; widths[] is free
        if (threadIdx.x < n) {
            const uint32_t t = base + threadIdx.x;
            const uint32_t width = blob[p.off_bits + t];
            const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
            // a damaged token is skipped rather than read out of bounds
            const bool good = token_in_range(p, width, po);
            widths[threadIdx.x] = good ? (uint8_t)width : 0;
        }
        __syncthreads();
        for (uint32_t b = 2; b <= 8; ++b) {
            bool any = false;                              // uniform: depends on widths[] only
            for (uint32_t k = 0; k < n; ++k) {
                if (widths[k] != b) continue;
                any = true;
                if (run < p.runs) {
                    const uint32_t t = base + k;
                    const uint64_t po = reinterpret_cast<const uint64_t *>(blob + p.off_pay_off)[t];
                    const uint32_t left = p.hidden - run * kRun;
                    const uint32_t *src_row = reinterpret_cast<const uint32_t *>(blob + p.off_payload + po);
                    uint32_t *mine = bins + (threadIdx.x & (kCopies - 1u)) * kCopyStride;
                    if (__builtin_amdgcn_ballot_w64(left < 32u) == 0) count_run_any<false>(b, src_row, run, left, mine);
                    else count_run_any<true>(b, src_row, run, left, mine);
                }
            }
            if (!any) continue;
            __syncthreads();
            for (uint32_t c = threadIdx.x; c < 256u; c += blockDim.x) {
                uint32_t s = 0;
#pragma unroll
                for (uint32_t j = 0; j < kCopies; ++j) s += bins[j * kCopyStride + c];
                acc[(b - 2u) * 256u + c] += s;
            }
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < kCopies * kCopyStride; i += blockDim.x) bins[i] = 0;
            __syncthreads();
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < 7u * 256u; i += blockDim.x)
        if (acc[i]) atomicAdd(mine_out + i, acc[i]);
}

int launch_code_hist(const Params &p, const Geometry &g, const void *d_blob, void *d_hist, void *stream) {
    hipLaunchKernelGGL(k_code_hist, dim3(p.tokens), dim3(g.block), 0, reinterpret_cast<hipStream_t>(stream), p,
                       static_cast<const uint8_t *>(d_blob), static_cast<uint32_t *>(d_hist));
    return (int)hipGetLastError();
}

int launch_code_pool(const Params &p, const Geometry &g, const EntropyLayout &e, const void *d_blob, void *d_counts,
                     void *stream) {
    hipLaunchKernelGGL(k_code_pool, dim3(e.pool_groups), dim3(g.block), 0, reinterpret_cast<hipStream_t>(stream), p,
                       static_cast<const uint8_t *>(d_blob), static_cast<uint32_t *>(d_counts), e.pool_tokens);
    return (int)hipGetLastError();
}

}  // namespace tsq
