// Device-side building blocks of the row kernels (gfx950, wave64).
//
// Data ownership inside a workgroup: the row of `hidden` 16-bit values is cut
// into runs of 32 consecutive elements; lane r of the workgroup owns run r.
// A run is 64 bytes of input (4 pieces of 16 B), 8 dwords of packed magnitude
// bytes, and exactly b dwords of packed b-bit codes, so packing never crosses
// lanes.  Rows travel between HBM and the lanes through LDS: global accesses
// are 16 B per lane with consecutive lanes on consecutive addresses, and the
// LDS copy of run r starts at dword r*kRunLdsDw (padded against bank conflicts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsq_internal.hpp"
#include "tsq_ranges.hpp"

namespace tsq {

constexpr int kF16 = 0, kBF16 = 1;
constexpr int kModeLsb = 0;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // 16 bytes at a 4-byte aligned address

__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, a) - __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t,
                              __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_ashr15_i16(uint32_t a) {
    return __builtin_bit_cast(uint32_t, (i16x2)(__builtin_bit_cast(i16x2, a) >> 15));
}

// ---------------------------------------------------------------- wave / block collectives

// DPP controls (gfx9): quad_perm [1,0,3,2] and [2,3,0,1], mirror inside 8 lanes, mirror inside a
// row of 16 lanes, shift right inside a row by n.
constexpr int kDppQuadXor1 = 0xB1, kDppQuadXor2 = 0x4E, kDppHalfMirror = 0x141, kDppRowMirror = 0x140;
constexpr int kDppRowShr = 0x110;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t lane_value(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

// A value that is the same in every lane, moved to a scalar register (frees a vector register and
// lets the arithmetic that follows run on the scalar unit).
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// The B payload words of a run of 32 b-bit codes, as few memory instructions as B allows (16, 8 and 4
// bytes; a payload row is only 4-byte aligned, which is all that these need on this hardware).  A lane that
// takes one word at a time makes the memory pipeline walk the cache lines under a wave's runs B times.
typedef uint32_t Words4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t Words2 __attribute__((ext_vector_type(2), aligned(4)));
template <int B>
__device__ __forceinline__ void load_run_words(const uint32_t *src, uint32_t (&d)[B]) {
    int k = 0;
#pragma unroll
    for (; k + 4 <= B; k += 4) {
        const Words4 v = *reinterpret_cast<const Words4 *>(src + k);
        d[k] = v.x; d[k + 1] = v.y; d[k + 2] = v.z; d[k + 3] = v.w;
    }
    if (k + 2 <= B) {
        const Words2 v = *reinterpret_cast<const Words2 *>(src + k);
        d[k] = v.x; d[k + 1] = v.y;
        k += 2;
    }
    if (k < B) d[k] = src[k];
}
template <int B>
__device__ __forceinline__ void store_run_words(uint32_t *dst, const uint32_t (&d)[B]) {
    int k = 0;
#pragma unroll
    for (; k + 4 <= B; k += 4) {
        Words4 v; v.x = d[k]; v.y = d[k + 1]; v.z = d[k + 2]; v.w = d[k + 3];
        *reinterpret_cast<Words4 *>(dst + k) = v;
    }
    if (k + 2 <= B) {
        Words2 v; v.x = d[k]; v.y = d[k + 1];
        *reinterpret_cast<Words2 *>(dst + k) = v;
        k += 2;
    }
    if (k < B) dst[k] = d[k];
}

// Reductions over the 64 lanes of a wave; the result is uniform.  Four DPP steps leave the
// total of each row of 16 lanes in all of its lanes; the four row totals are combined as scalars.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    uint32_t n;
    n = dpp<kDppQuadXor1>(v);   v = n > v ? n : v;
    n = dpp<kDppQuadXor2>(v);   v = n > v ? n : v;
    n = dpp<kDppHalfMirror>(v); v = n > v ? n : v;
    n = dpp<kDppRowMirror>(v);  v = n > v ? n : v;
    const uint32_t a = lane_value(v, 0), b = lane_value(v, 16), c = lane_value(v, 32), d = lane_value(v, 48);
    const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
    v += dpp<kDppQuadXor1>(v);
    v += dpp<kDppQuadXor2>(v);
    v += dpp<kDppHalfMirror>(v);
    v += dpp<kDppRowMirror>(v);
    return lane_value(v, 0) + lane_value(v, 16) + lane_value(v, 32) + lane_value(v, 48);
}
// Inclusive prefix sum over the lanes of a wave, in lane order: four shifts inside the rows of 16
// lanes, then the last lane of row 0 (2) is added to row 1 (3), and the last lane of row 1, by then
// the total of rows 0 and 1, to rows 2 and 3.
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
    v += dpp<kDppRowShr + 1>(v);    // lanes without a source inside their row add 0
    v += dpp<kDppRowShr + 2>(v);
    v += dpp<kDppRowShr + 4>(v);
    v += dpp<kDppRowShr + 8>(v);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kDppRowBcast15, 0xA, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kDppRowBcast31, 0xC, 0xF, false);
    return v;
}

// Exclusive prefix sum of v over the threads of the block, in thread order.
// scr: kMaxWaves dwords of LDS not in use by anything else until the next barrier.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *scr) {
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const uint32_t inc = wave_incl_scan_u32(v);
    if (lane == 63) scr[wv] = inc;
    __syncthreads();
    uint32_t base = 0;
    for (uint32_t w = 0; w < wv; ++w) base += scr[w];
    return base + inc - v;
}

// A window of `bytes` bytes of device memory at a uniform address as a raw buffer resource (stride 0,
// the untyped 32-bit format word of this chip family): stores beyond the window are dropped by
// the hardware.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_window(void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, 0x00027000);
}
// 16 bytes to window + offset (4-byte aligned) with device-scope write-through (cache policy sc1):
// the line does not stay dirty in the L2.
__device__ __forceinline__ void store_quad_through(__amdgpu_buffer_rsrc_t window, uint32_t offset, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, window, (int)offset, 0, 16);
}

// ---------------------------------------------------------------- row staging

// Row movement HBM -> registers -> LDS, private to each wave: wave w moves the 4 KB of the row
// that its own lanes own (runs 64w .. 64w+63): four coalesced loads of 16 B per lane, then four
// 16-byte LDS writes in the run layout.  Since a wave only reads back what it wrote itself and
// the LDS operations of one wave execute in order, the row needs no workgroup barrier.
struct RowPart { uint32_t w[16]; };   // the four 16-byte pieces a lane moves, as scalars

// src is uniform and points into device memory (it may come out of a table of pointers, which hides
// that from the compiler): the loads name the global address space, so that they are ordinary
// vector memory loads and not loads that might also hit LDS or scratch.
typedef const __attribute__((address_space(1))) uint8_t *GlobalBytes;
// spread: 16 to fetch the row; 0 makes every lane fetch the row's first piece (for a caller that must issue
// the loads but has no row to fetch: one cache line instead of a whole row)
template <bool FULL = false>
__device__ __forceinline__ void fetch_row_part(const uint4 *__restrict__ src, uint32_t pieces, RowPart &pre,
                                               uint32_t spread = 16u) {
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
    const GlobalBytes base = (GlobalBytes)src;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t q = 256u * wv + 64u * k + lane;
        uint32_t x = 0, y = 0, z = 0, w = 0;
        if (FULL || q < pieces) {
            // the input is read once: streaming load
            const u32x4 v = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4 *)(base + spread * q));
            x = v.x; y = v.y; z = v.z; w = v.w;
        }
        pre.w[4 * k] = x; pre.w[4 * k + 1] = y; pre.w[4 * k + 2] = z; pre.w[4 * k + 3] = w;
    }
}
__device__ __forceinline__ void write_row_part(uint32_t *lrow, uint32_t runs, const RowPart &pre) {
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t q = 256u * wv + 64u * k + lane;
        if (q < 4 * runs)
            *reinterpret_cast<uint4 *>(lrow + (q >> 2) * kRunLdsDw + (q & 3) * 4) =
                make_uint4(pre.w[4 * k], pre.w[4 * k + 1], pre.w[4 * k + 2], pre.w[4 * k + 3]);
    }
}

// ---------------------------------------------------------------- Eq. (ts) on one run

// The inlier part T_below of a run in the form the quantizer consumes:
//   bf16: 32 binary32 values;
//   fp16: 16 dwords of packed half-precision values (the multiply reads them directly
//         through v_fma_mix_f32).
// The values keep their sign (the multiply takes the magnitude through its source modifier, the
// packing takes the sign bit from here), outlier slots hold +0 in both forms.
template <int DT> struct Mags;
template <> struct Mags<kBF16> { float v[32]; };
template <> struct Mags<kF16> { uint32_t v[16]; };

// ((w & inl) & 0xFFFF) << 16 in one SDWA instruction.  A VALU result written with a partial
// dst_sel must not be read by the very next VALU instruction on gfx950: the s_nop provides the
// wait state, since the compiler cannot see into the asm statement.
__device__ __forceinline__ float masked_low_half_as_bf16(uint32_t w, uint32_t inl) {
    uint32_t d;
    asm("v_and_b32_sdwa %0, %1, %2 dst_sel:WORD_1 dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:WORD_0\n\ts_nop 0"
        : "=v"(d)
        : "v"(w), "v"(inl));
    return __uint_as_float(d);
}
// max(|a|, |b|, c) of binary32 values in one instruction; c >= 0.  For finite values the order of the
// magnitudes is the order of their bit patterns, so the result is the pattern of the largest magnitude.
__device__ __forceinline__ uint32_t max3_magnitude(float a, float b, uint32_t c) {
    uint32_t d;
    asm("v_max3_f32 %0, |%1|, |%2|, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
// Any boolean function of three words in one instruction (v_bitop3_b32): bit i of the result is bit
// (4 a_i + 2 b_i + c_i) of TABLE, i.e. TABLE is the function applied to a = 0xF0, b = 0xCC, c = 0xAA.
// On gfx950 it issues at the rate of a plain and / or (twice the rate of v_and_or_b32, v_or3_b32, v_bfi_b32).
template <int TABLE>
__device__ __forceinline__ uint32_t bitop3(uint32_t a, uint32_t b, uint32_t c) {
    return (uint32_t)__builtin_amdgcn_bitop3_b32((int)a, (int)b, (int)c, TABLE);
}
constexpr int kAndOr = (0xF0 & 0xCC) | 0xAA;            // (a & b) | c
constexpr int kSelect = (0xF0 & 0xCC) | (~0xF0 & 0xAA & 0xFF);   // a ? b : c, bit by bit
constexpr int kOrAnd = (0xF0 | 0xCC) & 0xAA;            // (a | b) & c
constexpr int kAnd3 = 0xF0 & 0xCC & 0xAA;               // a & b & c

// bits `sel` of keep into old
__device__ __forceinline__ uint32_t bit_insert(uint32_t sel, uint32_t keep, uint32_t old) {
    return bitop3<kAndOr>(keep, sel, old);
}

// Threshold splitting (Eq. (ts)) of the 32 elements a lane owns, on the 16-bit magnitude
// patterns: for fp16 and bf16 alike the pattern of |x| grows with |x|, and the patterns of Inf
// and NaN lie above every finite one, so
//   !(|x| < tau)  <=>  (pattern & 0x7FFF) >= thr,
// thr being the smallest pattern whose value is >= tau (computed on the host).
//   mg        : T_below of the run (see Mags)
//   omask     : outlier flags in column order, bit j = element j
//   amax_bits : binary32 bit pattern of the largest inlier magnitude of the run (only if WANT_MAX)
// Per pair of elements: and, subtract, packed arithmetic shift, bit-field insert into the flags;
// then bf16: two masked widenings and one three-way max (7 instructions), fp16: two ands and one
// packed max (7).  The subtract is a plain 32-bit one (it issues at twice the rate of the packed
// 16-bit form): with g = thr + 0x7FFF = (thr - 1) | 0x8000 in both halves, g - pattern leaves in
// each half 0x8000 + (thr - 1 - pattern), which is never negative (pattern <= 0x7FFF, thr >= 1),
// so nothing is borrowed from the upper half, and whose bit 15 is set exactly for the inliers.
// The flags of a pair are 16 bits apart in `inl`, so the pairs 0-7 and 8-15 are collected in two
// words (low element at bit 2i', high element at bit 17+2i', i' = i mod 8) that are folded into
// column order at the end.
template <int DT, bool WANT_MAX>
__device__ __forceinline__ void split_regs(const uint32_t (&w)[16], uint32_t thr_pk, Mags<DT> &mg, uint32_t &omask,
                                           uint32_t &amax_bits) {
    uint32_t im_a = 0, im_b = 0;           // inlier flags of the pairs 0-7 / 8-15, collected bit by bit
    const uint32_t guard_pk = thr_pk + 0x7FFF7FFFu;
    if constexpr (DT == kBF16) {
        uint32_t mx = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t absw = w[i] & 0x7FFF7FFFu;
            const uint32_t inl = pk_ashr15_i16(guard_pk - absw);  // 0xFFFF where |x| < tau
            const float lo = masked_low_half_as_bf16(w[i], inl);
            const float hi = __uint_as_float(bitop3<kAnd3>(w[i], inl, 0xFFFF0000u));
            mg.v[2 * i] = lo;
            mg.v[2 * i + 1] = hi;
            if (WANT_MAX) mx = max3_magnitude(lo, hi, mx);
            if (i < 8) im_a = bit_insert(0x00020001u << (2 * i), inl, im_a);
            else im_b = bit_insert(0x00020001u << (2 * (i - 8)), inl, im_b);
        }
        amax_bits = mx;
    } else {
        uint32_t mx = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t absw = w[i] & 0x7FFF7FFFu;
            const uint32_t inl = pk_ashr15_i16(guard_pk - absw);
            mg.v[i] = w[i] & inl;
            if (WANT_MAX) mx = pk_max_u16(mx, absw & inl);
            if (i < 8) im_a = bit_insert(0x00020001u << (2 * i), inl, im_a);
            else im_b = bit_insert(0x00020001u << (2 * (i - 8)), inl, im_b);
        }
        const uint32_t m16 = (mx & 0xFFFFu) > (mx >> 16) ? (mx & 0xFFFFu) : (mx >> 16);
        amax_bits = __float_as_uint((float)__builtin_bit_cast(_Float16, (unsigned short)m16));
    }
    // pairs 0-7: even columns sit in the low half already, the odd ones come down from the high half;
    // pairs 8-15: the odd columns sit in the high half already, the even ones go up
    const uint32_t im = ((im_a | (im_a >> 16)) & 0x0000FFFFu) | ((im_b | (im_b << 16)) & 0xFFFF0000u);
    omask = ~im;
}

// A run in the padded LDS row of the staged kernels.
__device__ __forceinline__ void load_run_padded(const uint32_t *lrun, uint32_t (&w)[16]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 q = *reinterpret_cast<const uint4 *>(lrun + 4 * k);
        w[4 * k] = q.x; w[4 * k + 1] = q.y; w[4 * k + 2] = q.z; w[4 * k + 3] = q.w;
    }
}
template <int DT, bool WANT_MAX>
__device__ __forceinline__ void split_run(const uint32_t *lrun, uint32_t thr_pk, Mags<DT> &mg, uint32_t &omask,
                                          uint32_t &amax_bits) {
    uint32_t w[16];
    load_run_padded(lrun, w);
    split_regs<DT, WANT_MAX>(w, thr_pk, mg, omask, amax_bits);
}

// Lane-private copy of a run in LDS, 16 dwords per lane, no padding: the four 16-byte chunks
// of lane r are stored in the order k ^ ((r >> 1) & 3), which spreads 8 neighbouring lanes
// over all 32 banks.
__device__ __forceinline__ void slot_write(uint32_t *slot, uint32_t r, const uint32_t (&w)[16]) {
    const uint32_t sw = (r >> 1) & 3u;
    uint32_t *base = slot + r * 16;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k)
        *reinterpret_cast<uint4 *>(base + ((k ^ sw) << 2)) = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
}
__device__ __forceinline__ void slot_read(const uint32_t *slot, uint32_t r, uint32_t (&w)[16]) {
    const uint32_t sw = (r >> 1) & 3u;
    const uint32_t *base = slot + r * 16;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        const uint4 q = *reinterpret_cast<const uint4 *>(base + ((k ^ sw) << 2));
        w[4 * k] = q.x; w[4 * k + 1] = q.y; w[4 * k + 2] = q.z; w[4 * k + 3] = q.w;
    }
}
__device__ __forceinline__ uint16_t slot_raw(const uint32_t *slot, uint32_t r, uint32_t j) {
    const uint32_t d = j >> 1;
    const uint32_t pos = r * 16 + ((((d >> 2) ^ ((r >> 1) & 3u)) << 2) | (d & 3u));
    return reinterpret_cast<const uint16_t *>(slot)[2 * pos + (j & 1u)];
}

template <int DT>
__device__ __forceinline__ float widen_lo(uint32_t w) {
    if (DT == kBF16) return __uint_as_float(w << 16);
    return (float)__builtin_bit_cast(_Float16, (unsigned short)(w & 0xFFFFu));
}
template <int DT>
__device__ __forceinline__ float widen_hi(uint32_t w) {
    if (DT == kBF16) return __uint_as_float(w & 0xFFFF0000u);
    return (float)__builtin_bit_cast(_Float16, (unsigned short)(w >> 16));
}
template <int DT>
__device__ __forceinline__ float widen16(uint32_t pattern) {
    return widen_lo<DT>(pattern & 0xFFFFu);
}

// ---------------------------------------------------------------- Eq. (Proposed) on one run

// fl(|a| * r) for the low / high half-precision value of a packed pair: v_fma_mix_f32 widens the
// half exactly and rounds the product once, which is the binary32 product of the widened value.
__device__ __forceinline__ float mul_f16_lo(uint32_t pk, float r) {
    float d;
    asm("v_fma_mix_f32 %0, |%1|, %2, 0 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pk), "v"(r));
    return d;
}
__device__ __forceinline__ float mul_f16_hi(uint32_t pk, float r) {
    float d;
    asm("v_fma_mix_f32 %0, |%1|, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pk), "v"(r));
    return d;
}

// m = rint(|a| * r), one byte per element, element 4g+k in byte k of m[g]: one multiply and one
// convert per element.  The rounding is done by v_cvt_pk_u8_f32 itself, which converts with
// round-to-nearest-even (checked on gfx950 on exact halves 0.5, 1.5, 2.5, ... and pinned by the
// tie rows of the parity tests) and saturates at 255.  A clamp min(., Q) to the code range never
// binds: a <= amax and r = fl(Q/amax) give a*r <= Q*(1+2^-24)^2 < Q + 1/2, so rint already
// yields at most Q.
template <int DT>
__device__ __forceinline__ void quantize_run(const Mags<DT> &mg, float r, uint32_t (&m)[8]) {
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        uint32_t acc = 0;
        if constexpr (DT == kBF16) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                acc = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fabsf(mg.v[4 * g + k]) * r, k, acc);
        } else {
            acc = __builtin_amdgcn_cvt_pk_u8_f32(mul_f16_lo(mg.v[2 * g], r), 0, acc);
            acc = __builtin_amdgcn_cvt_pk_u8_f32(mul_f16_hi(mg.v[2 * g], r), 1, acc);
            acc = __builtin_amdgcn_cvt_pk_u8_f32(mul_f16_lo(mg.v[2 * g + 1], r), 2, acc);
            acc = __builtin_amdgcn_cvt_pk_u8_f32(mul_f16_hi(mg.v[2 * g + 1], r), 3, acc);
        }
        m[g] = acc;
    }
}

__device__ __forceinline__ uint32_t sum_squares_run(const uint32_t (&m)[8]) {
    uint32_t s = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) s = __builtin_amdgcn_udot4(m[g], m[g], s, false);
    return s;
}

// sum over the run of | (m0 >> sh) - mi |, bytewise
__device__ __forceinline__ uint32_t sad_run(const uint32_t (&m0)[8], const uint32_t (&mi)[8], uint32_t sh) {
    const uint32_t keep = (0xFFu >> sh) * 0x01010101u;
    uint32_t s = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) s = __builtin_amdgcn_sad_u8((m0[g] >> sh) & keep, mi[g], s);
    return s;
}

// Algorithm 1's stopping test, the same fixed sequence of fp64 operations on every lane:
//   LSB:      (double)sad > (double)budget * (double)H
//   REL_RMS:  L = (double)Q0 * (double)sad; L *= L; R = (double)budget * (double)Qi; R *= R; R *= (double)H;
//             R *= (double)ss0; L > R
// rhs is the part of the right-hand side that the host computed in that sequence (Params::test_rhs): all of it
// (LSB), or R before its last factor (REL_RMS).
__device__ __forceinline__ bool violates(int mode, double rhs, uint32_t Q0, uint32_t sad, uint32_t ss0) {
    if (mode == kModeLsb) return (double)sad > rhs;
    double L = (double)Q0 * (double)sad;
    L *= L;
    const double R = rhs * (double)ss0;
    return L > R;
}

constexpr float kAmaxFloor = 0x1p-100f;  // below it Q/amax may overflow binary32: row is coded as zeros

__device__ __forceinline__ float level_count(uint32_t width) { return (float)((1u << (width - 1)) - 1u); }

// ---------------------------------------------------------------- bit packing of one run

// The sign bits of elements 4g .. 4g+3 in bit 7 of bytes 0 .. 3 (the other bits are whatever the
// top bytes of the values hold), and-ed with `keep`.
template <int DT>
__device__ __forceinline__ uint32_t sign_bytes_and(const Mags<DT> &mg, int g, uint32_t keep) {
    if constexpr (DT == kBF16) {
        // the top byte of two binary32 values per v_perm_b32: bytes 0, 1 from the first pair, 2, 3 from the second
        const uint32_t p01 = __builtin_amdgcn_perm(__float_as_uint(mg.v[4 * g + 1]), __float_as_uint(mg.v[4 * g]), 0x0c0c0703u);
        const uint32_t p23 = __builtin_amdgcn_perm(__float_as_uint(mg.v[4 * g + 3]), __float_as_uint(mg.v[4 * g + 2]), 0x07030c0cu);
        return bitop3<kOrAnd>(p01, p23, keep);
    } else {
        // byte k <- high byte of element 4g+k
        return __builtin_amdgcn_perm(mg.v[2 * g + 1], mg.v[2 * g], 0x07050301u) & keep;
    }
}

// out[0..B) = the run's 32 codes, LSB first.  m: magnitude bytes; mg: the run's T_below (sign
// bits).  The sign is dropped where the magnitude is 0.
template <int B, int DT>
__device__ __forceinline__ void pack_regs(const uint32_t (&m)[8], const Mags<DT> &mg, uint32_t (&out)[B]) {
    constexpr uint32_t K = (1u << (B - 1)) - 1u;
    uint64_t acc = 0;
    int filled = 0, od = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const uint32_t mb = m[g];
        const uint32_t nzb = mb + K * 0x01010101u;                       // bit B-1 of each byte: m > 0
        uint32_t code;
        if (B == 8) {
            code = bitop3<kAndOr>(sign_bytes_and<DT>(mg, g, nzb), 0x80808080u, mb);
        } else {
            const uint32_t sg = sign_bytes_and<DT>(mg, g, 0x80808080u) >> (8 - B);   // sign now at bit B-1 of each byte
            code = bitop3<kAndOr>(sg, nzb, mb);
        }
        uint32_t chunk;
        if (B == 8) {
            chunk = code;
        } else {
            // two codes per 16-bit half side by side, then the two halves side by side: right shifts and
            // three-input bit operations only (left shifts and the fused shift-or forms issue at half rate)
            constexpr uint32_t F = (1u << B) - 1u, M = (1u << (2 * B)) - 1u;
            const uint32_t t = bitop3<kAndOr>(code >> (8 - B), (F << B) * 0x00010001u, code & (F * 0x00010001u));
            chunk = bitop3<kSelect>(M, t, t >> (16 - 2 * B));
        }
        acc |= (uint64_t)chunk << filled;
        filled += 4 * B;
        if (filled >= 32) {
            out[od++] = (uint32_t)acc;
            acc >>= 32;
            filled -= 32;
        }
    }
}

// Inverse of pack_regs followed by Eq. (dequnt) for the inliers: 32 codes ->
// 16 dwords of 16-bit values sign * (m * s), rounded to nearest even.
template <int DT>
__device__ __forceinline__ uint32_t narrow2(float lo, float hi) {
    if (DT == kBF16) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
    const unsigned short l = __builtin_bit_cast(unsigned short, (_Float16)lo);
    const unsigned short h = __builtin_bit_cast(unsigned short, (_Float16)hi);
    return (uint32_t)l | ((uint32_t)h << 16);
}

template <int B>
__device__ __forceinline__ float decode_one(const uint32_t (&d)[B], int j, float s) {
    const int off = j * B;
    const int k = off >> 5, sh = off & 31;
    uint32_t code = d[k] >> sh;
    if (sh + B > 32) code |= d[k + 1 < B ? k + 1 : k] << (32 - sh);
    const uint32_t mag = code & ((1u << (B - 1)) - 1u);
    const uint32_t neg = (code >> (B - 1)) & 1u;
    const float v = (float)mag * s;
    return __uint_as_float(__float_as_uint(v) | (neg << 31));
}

template <int DT, int B>
__device__ __forceinline__ void unpack_run(const uint32_t (&d)[B], float s, uint32_t (&o)[16]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) o[i] = narrow2<DT>(decode_one<B>(d, 2 * i, s), decode_one<B>(d, 2 * i + 1, s));
}

// LDS scratch of the staged row kernels (behind the row): four reduce areas | scan area
constexpr uint32_t kScrScan = 4 * 2 * kMaxWaves;

__device__ __forceinline__ uint32_t row_bytes(uint32_t H, uint32_t b) { return payload_row_bytes(H, b); }
// A token of width b whose payload starts at byte po of the payload section (see tsq_ranges.hpp).
__device__ __forceinline__ bool token_in_range(const Params &p, uint32_t b, uint64_t po) {
    return payload_span_ok(p.hidden, p.payload_capacity, b, po);
}

// ---------------------------------------------------------------- Algorithm 1 for the token of this block

struct RowStats {
    float amax;           // inlier absmax of the token
    uint32_t cnt;         // outliers in the token
    uint32_t cnt_before;  // ... in the waves before this one
    uint32_t cnt_wave;    // ... in this wave
};
struct Choice {
    uint32_t width;       // b_t
    float scale;          // s_t = amax / Q_{b_t} (0 for a row coded as zeros)
};

// Workgroup barrier that orders LDS accesses only (what the cross-wave reductions need): a wave
// does not wait for its outstanding device-memory operations here, in particular not for a row
// that is on its way into LDS.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- block collectives for NW waves (known at compile time) ----
// A reduce area is 2*kMaxWaves dwords; slot w = wave w's first value, kMaxWaves + w its second.
// The caller rotates over four areas, so a wave that is one barrier ahead never overwrites
// values another wave still has to read.

// max of mx, sum of sm over the block; pre = sum of sm over the waves before this one, own = over this wave
template <int NW>
__device__ __forceinline__ void block_max_sum_prefix(uint32_t &mx, uint32_t &sm, uint32_t &pre, uint32_t &own,
                                                     uint32_t *red) {
    mx = wave_max_u32(mx);
    sm = wave_sum_u32(sm);
    own = sm;
    pre = 0;
    if (NW == 1) return;
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) { red[wv] = mx; red[kMaxWaves + wv] = sm; }
    lds_barrier();
    uint32_t M = 0, S = 0, P = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t a = red[w], b = red[kMaxWaves + w];
        M = a > M ? a : M;
        S += b;
        P += (uint32_t)w < wv ? b : 0u;
    }
    mx = uniform(M); sm = uniform(S); pre = uniform(P);
}
template <int NW>
__device__ __forceinline__ void block_sum2_nw(uint32_t &x, uint32_t &y, uint32_t *red) {
    x = wave_sum_u32(x);
    y = wave_sum_u32(y);
    if (NW == 1) return;
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) { red[wv] = x; red[kMaxWaves + wv] = y; }
    lds_barrier();
    uint32_t X = 0, Y = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { X += red[w]; Y += red[kMaxWaves + w]; }
    x = uniform(X); y = uniform(Y);
}
template <int NW>
__device__ __forceinline__ void block_sum1_nw(uint32_t &x, uint32_t *red) {
    x = wave_sum_u32(x);
    if (NW == 1) return;
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) red[wv] = x;
    lds_barrier();
    uint32_t X = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) X += red[w];
    x = uniform(X);
}

// Inlier absmax and outlier count of the token of this block (one barrier).  ring: four reduce
// areas; turn: running count of reductions; lanes that own no run pass omask = 0, amax_bits = 0.
template <int NW>
__device__ __forceinline__ RowStats reduce_row_stats(uint32_t omask, uint32_t amax_bits, uint32_t *ring,
                                                     uint32_t &turn) {
    uint32_t mx = amax_bits;              // non-negative binary32 patterns order like unsigned integers
    uint32_t cnt = (uint32_t)__builtin_popcount(omask);
    RowStats st;
    block_max_sum_prefix<NW>(mx, cnt, st.cnt_before, st.cnt_wave, ring + (turn++ & 3u) * 2 * kMaxWaves);
    st.amax = __uint_as_float(mx);
    st.cnt = cnt;
    return st;
}

// The same with the wave's outlier count already summed by the caller.
template <int NW>
__device__ __forceinline__ RowStats reduce_row_stats_counted(uint32_t amax_bits, uint32_t cnt_wave, uint32_t *ring,
                                                             uint32_t &turn) {
    RowStats st;
    uint32_t mx = wave_max_u32(amax_bits), cnt = cnt_wave, before = 0;
    if (NW > 1) {
        uint32_t *red = ring + (turn++ & 3u) * 2 * kMaxWaves;
        const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
        if (lane == 0) { red[wv] = mx; red[kMaxWaves + wv] = cnt_wave; }
        lds_barrier();
        uint32_t M = 0, S = 0, P = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t a = red[w], b = red[kMaxWaves + w];
            M = a > M ? a : M;
            S += b;
            P += (uint32_t)w < wv ? b : 0u;
        }
        mx = uniform(M); cnt = uniform(S); before = uniform(P);
    } else {
        ++turn;
    }
    st.amax = __uint_as_float(mx);
    st.cnt = cnt;
    st.cnt_before = before;
    st.cnt_wave = cnt_wave;
    return st;
}

// Algorithm 1 for the token of this block, given its inlier absmax.  live: false for lanes that
// own no run (they compute on a copy of run 0 and are left out of every sum).  On return m holds
// the magnitude bytes of the run at the chosen width.
// The divisions of Eq. (Proposed) for all allowed widths are one division per wave: lane k < 8
// computes Q_k / amax, lane 8 + k computes amax / Q_k (the scale, should width k be chosen).
template <int DT, int NW>
__device__ __forceinline__ Choice search_width(const Params &p, const Mags<DT> &af, float amax, bool live,
                                               uint32_t *ring, uint32_t &turn, uint32_t (&m)[8]) {
    const uint32_t lane = threadIdx.x & 63;
    float quot = 0.0f;
    if ((lane & 7u) < p.n_widths && lane < 16u && amax >= kAmaxFloor) {
        const float q = level_count(width_at(p, lane & 7u));
        quot = lane < 8u ? q / amax : amax / q;
    }
    const uint32_t quot_bits = __float_as_uint(quot);

    const uint32_t b0 = width_at(p, 0);
    const uint32_t Q0 = (1u << (b0 - 1)) - 1u;
    quantize_run<DT>(af, __uint_as_float(__builtin_amdgcn_readlane(quot_bits, 0)), m);
    uint32_t sel = b0, sel_i = 0;
    if (p.n_widths > 1) {
        uint32_t m0[8];
#pragma unroll
        for (int g = 0; g < 8; ++g) m0[g] = m[g];
        uint32_t ss0 = live ? sum_squares_run(m0) : 0u;
        for (uint32_t i = 1; i < p.n_widths; ++i) {
            const uint32_t bi = width_at(p, i);
            uint32_t mi[8];
            quantize_run<DT>(af, __uint_as_float(__builtin_amdgcn_readlane(quot_bits, (int)i)), mi);
            uint32_t sad = live ? sad_run(m0, mi, b0 - bi) : 0u;
            uint32_t *red = ring + (turn++ & 3u) * 2 * kMaxWaves;
            if (i == 1) block_sum2_nw<NW>(sad, ss0, red); else block_sum1_nw<NW>(sad, red);
            // (Algorithm 1 as printed returns the quantization that failed the test; the default keeps
            // the last one that passed)
            const bool failed = violates(p.mode, p.test_rhs[i], Q0, sad, ss0);
            if (failed && !p.return_failing) break;
            sel = bi;
            sel_i = i;
#pragma unroll
            for (int g = 0; g < 8; ++g) m[g] = mi[g];
            if (failed) break;
        }
    }
    Choice c;
    c.width = sel;
    c.scale = __uint_as_float(__builtin_amdgcn_readlane(quot_bits, (int)(8u + sel_i)));
    return c;
}

// The 128-byte header at the start of the blob (written by one thread).
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

}  // namespace tsq
