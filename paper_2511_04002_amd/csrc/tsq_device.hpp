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

namespace tsq {

constexpr int kF16 = 0, kBF16 = 1;
constexpr int kModeLsb = 0;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));

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
// Inclusive prefix sum over the lanes of a wave, in lane order.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
    v += dpp<kDppRowShr + 1>(v);    // lanes without a source inside their row add 0
    v += dpp<kDppRowShr + 2>(v);
    v += dpp<kDppRowShr + 4>(v);
    v += dpp<kDppRowShr + 8>(v);
    const uint32_t r0 = lane_value(v, 15), r1 = lane_value(v, 31), r2 = lane_value(v, 47);
    const uint32_t row = (threadIdx.x & 63) >> 4;
    return v + (row > 0 ? r0 : 0u) + (row > 1 ? r1 : 0u) + (row > 2 ? r2 : 0u);
}

// Cross-wave step of the block reductions.  A reduce area is 2*kMaxWaves dwords of LDS: slot w
// holds wave w's first value, slot kMaxWaves + w its second.  Slots of waves that do not exist
// must hold 0 (clear_reduce_areas), so that whole quads of slots can be read with one 16-byte
// load each; 0 is the identity of both max and sum on unsigned values.
__device__ __forceinline__ void clear_reduce_areas(uint32_t *scratch) {
    if (threadIdx.x < 4 * kMaxWaves) scratch[threadIdx.x] = 0;
}
__device__ __forceinline__ uint32_t max4(const uint4 v, uint32_t m) {
    const uint32_t a = v.x > v.y ? v.x : v.y, b = v.z > v.w ? v.z : v.w;
    const uint32_t c = a > b ? a : b;
    return c > m ? c : m;
}

// Every thread gets max over the block of mx and sum over the block of sm.
// red: a reduce area; consecutive calls must alternate between two such areas.
__device__ __forceinline__ void block_max_sum(uint32_t &mx, uint32_t &sm, uint32_t *red) {
    mx = wave_max_u32(mx);
    sm = wave_sum_u32(sm);
    const uint32_t nw = blockDim.x >> 6;
    if (nw == 1) return;
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) { red[wv] = mx; red[kMaxWaves + wv] = sm; }
    __syncthreads();
    uint32_t M = 0, S = 0;
    for (uint32_t q = 0; 4 * q < nw; ++q) {
        const uint4 a = reinterpret_cast<const uint4 *>(red)[q];
        const uint4 b = reinterpret_cast<const uint4 *>(red + kMaxWaves)[q];
        M = max4(a, M);
        S += (b.x + b.y) + (b.z + b.w);
    }
    mx = M;
    sm = S;
}
__device__ __forceinline__ void block_sum2(uint32_t &x, uint32_t &y, uint32_t *red) {
    x = wave_sum_u32(x);
    y = wave_sum_u32(y);
    const uint32_t nw = blockDim.x >> 6;
    if (nw == 1) return;
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) { red[wv] = x; red[kMaxWaves + wv] = y; }
    __syncthreads();
    uint32_t X = 0, Y = 0;
    for (uint32_t q = 0; 4 * q < nw; ++q) {
        const uint4 a = reinterpret_cast<const uint4 *>(red)[q];
        const uint4 b = reinterpret_cast<const uint4 *>(red + kMaxWaves)[q];
        X += (a.x + a.y) + (a.z + a.w);
        Y += (b.x + b.y) + (b.z + b.w);
    }
    x = X;
    y = Y;
}
__device__ __forceinline__ void block_sum1(uint32_t &x, uint32_t *red) {
    x = wave_sum_u32(x);
    const uint32_t nw = blockDim.x >> 6;
    if (nw == 1) return;
    const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) red[wv] = x;
    __syncthreads();
    uint32_t X = 0;
    for (uint32_t q = 0; 4 * q < nw; ++q) {
        const uint4 a = reinterpret_cast<const uint4 *>(red)[q];
        X += (a.x + a.y) + (a.z + a.w);
    }
    x = X;
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

// ---------------------------------------------------------------- row staging

// HBM -> LDS, coalesced: slot p of the LDS row holds 16-byte piece p (zeros past the row's end).
__device__ __forceinline__ void stage_row(const uint4 *__restrict__ src, uint32_t pieces, uint32_t runs,
                                          uint32_t *lrow) {
    uint4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t p = threadIdx.x + k * blockDim.x;
        v[k] = make_uint4(0, 0, 0, 0);
        if (p < pieces) v[k] = src[p];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t p = threadIdx.x + k * blockDim.x;
        if (p < 4 * runs) *reinterpret_cast<uint4 *>(lrow + (p >> 2) * kRunLdsDw + (p & 3) * 4) = v[k];
    }
}

// ---------------------------------------------------------------- Eq. (ts) on one run

// Threshold splitting of the 32 elements a lane owns, on the 16-bit magnitude
// patterns: for fp16 and bf16 alike the pattern of |x| grows with |x|, and the
// patterns of Inf and NaN lie above every finite one, so
//   !(|x| < tau)  <=>  (pattern & 0x7FFF) >= thr,
// thr being the smallest pattern whose value is >= tau (computed on the host).
//   apk   : |x| patterns of the inliers, 0 at outlier slots (|T_below|)
//   omask : outlier flags; bit i = element 2i, bit 16+i = element 2i+1
//   amax  : running maximum of the inlier patterns, both halves (only if WANT_MAX)
// Six instructions per pair of elements: and, packed subtract, packed arithmetic shift
// (the borrow of pattern - thr marks the inliers), and, packed max, bit-field insert.
template <bool WANT_MAX>
__device__ __forceinline__ void split_regs(const uint32_t (&w)[16], uint32_t thr_pk, uint32_t (&apk)[16],
                                           uint32_t &omask, uint32_t &amax_pk) {
    uint32_t im = 0, mx = amax_pk;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t absw = w[i] & 0x7FFF7FFFu;
        const uint32_t inl = pk_ashr15_i16(pk_sub_u16(absw, thr_pk));  // 0xFFFF where |x| < tau
        const uint32_t a = absw & inl;
        apk[i] = a;
        if (WANT_MAX) mx = pk_max_u16(mx, a);
        const uint32_t sel = 0x00010001u << i;
        im = (inl & sel) | (im & ~sel);                                // v_bfi_b32
    }
    omask = ~im;
    amax_pk = mx;
}

// A run in the padded LDS row of the staged kernels.
__device__ __forceinline__ void load_run_padded(const uint32_t *lrun, uint32_t (&w)[16]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 q = *reinterpret_cast<const uint4 *>(lrun + 4 * k);
        w[4 * k] = q.x; w[4 * k + 1] = q.y; w[4 * k + 2] = q.z; w[4 * k + 3] = q.w;
    }
}
template <bool WANT_MAX>
__device__ __forceinline__ void split_run(const uint32_t *lrun, uint32_t thr_pk, uint32_t (&apk)[16],
                                          uint32_t &omask, uint32_t &amax_pk) {
    uint32_t w[16];
    load_run_padded(lrun, w);
    split_regs<WANT_MAX>(w, thr_pk, apk, omask, amax_pk);
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

// The inlier magnitudes of a run as binary32 (exact for both 16-bit formats); widened once and
// kept in registers, so that every quantization pass costs one multiply and one convert per element.
template <int DT>
__device__ __forceinline__ void widen_run(const uint32_t (&apk)[16], float (&af)[32]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        af[2 * i] = widen_lo<DT>(apk[i]);
        af[2 * i + 1] = widen_hi<DT>(apk[i]);
    }
}

// m = rint(a * r), one byte per element, element 4g+k in byte k of m[g].  The rounding is done by
// v_cvt_pk_u8_f32 itself, which converts with round-to-nearest-even (checked on gfx950 on exact
// halves 0.5, 1.5, 2.5, ... and pinned by the tie rows of the parity tests) and saturates at 255.
// A clamp min(., Q) to the code range never binds: a <= amax and r = fl(Q/amax) give
// a*r <= Q*(1+2^-24)^2 < Q + 1/2, so rint already yields at most Q.
__device__ __forceinline__ void quantize_run(const float (&af)[32], float r, uint32_t (&m)[8]) {
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        uint32_t acc = 0;
        acc = __builtin_amdgcn_cvt_pk_u8_f32(af[4 * g] * r, 0, acc);
        acc = __builtin_amdgcn_cvt_pk_u8_f32(af[4 * g + 1] * r, 1, acc);
        acc = __builtin_amdgcn_cvt_pk_u8_f32(af[4 * g + 2] * r, 2, acc);
        acc = __builtin_amdgcn_cvt_pk_u8_f32(af[4 * g + 3] * r, 3, acc);
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

// Algorithm 1's stopping test, the same fixed sequence of fp64 operations on every lane.
__device__ __forceinline__ bool violates(int mode, float budget, uint32_t H, uint32_t Q0, uint32_t Qi,
                                         uint32_t sad, uint32_t ss0) {
    if (mode == kModeLsb) return (double)sad > (double)budget * (double)H;
    double L = (double)Q0 * (double)sad;
    L *= L;
    double R = (double)budget * (double)Qi;
    R *= R;
    R *= (double)H;
    R *= (double)ss0;
    return L > R;
}

constexpr float kAmaxFloor = 0x1p-100f;  // below it Q/amax may overflow binary32: row is coded as zeros

__device__ __forceinline__ float level_count(uint32_t width) { return (float)((1u << (width - 1)) - 1u); }

// ---------------------------------------------------------------- bit packing of one run

// out[0..B) = the run's 32 codes, LSB first.  m: magnitude bytes; w: the run's
// raw input dwords (sign bits).  The sign is dropped where the magnitude is 0.
template <int B>
__device__ __forceinline__ void pack_regs(const uint32_t (&m)[8], const uint32_t (&w)[16], uint32_t (&out)[B]) {
    constexpr uint32_t K = (1u << (B - 1)) - 1u;
    uint64_t acc = 0;
    int filled = 0, od = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const uint32_t mg = m[g];
        // byte k <- high byte of element 4g+k (bit 7 of it is the sign)
        const uint32_t sg = __builtin_amdgcn_perm(w[2 * g + 1], w[2 * g], 0x07050301u);
        const uint32_t sgb = (B == 8) ? sg : (sg >> (8 - B));            // sign now at bit B-1 of each byte
        const uint32_t nzb = mg + K * 0x01010101u;                       // bit B-1 of each byte: m > 0
        const uint32_t code = mg | (sgb & nzb & (0x01010101u << (B - 1)));
        uint32_t chunk;
        if (B == 8) {
            chunk = code;
        } else {
            constexpr uint32_t F = (1u << B) - 1u;
            const uint32_t t = (code & (F * 0x00010001u)) | ((code >> (8 - B)) & ((F << B) * 0x00010001u));
            chunk = (t & 0xFFFFu) | ((t >> 16) << (2 * B));
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

template <int B>
__device__ __forceinline__ void pack_run(const uint32_t (&m)[8], const uint32_t *lrun, uint32_t (&out)[B]) {
    uint32_t w[16];
    load_run_padded(lrun, w);
    pack_regs<B>(m, w, out);
}

// Inverse of pack_run followed by Eq. (dequnt) for the inliers: 32 codes ->
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

}  // namespace tsq
