// Admissibility of offsets and sizes that a kernel reads from memory it does not own (a blob, an
// entropy-coded blob, a workspace) before it uses them as addresses.  Plain integer predicates on
// plain values, written without sums of untrusted values (which could wrap), compiled for the
// device (the kernels call them) and for the host (tsq_check_* in tsq_api.hip evaluates them
// for tests that need no GPU).  Also here, for the same reason: the one piece of the entropy coder's
// arithmetic whose exactness rests on a rounding argument.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define TSQ_HD __host__ __device__ __forceinline__
#else
#define TSQ_HD inline
#endif

namespace tsq {

// bytes of one token's payload at width b: b bits per element, padded to a 4-byte multiple
TSQ_HD uint32_t payload_row_bytes(uint32_t hidden, uint32_t b) { return 4u * ((hidden * b + 31u) >> 5); }

// A token of width b whose payload starts at byte po of a payload section of `capacity` bytes:
// a width of the format, 4-byte aligned, and wholly inside the section.
TSQ_HD bool payload_span_ok(uint32_t hidden, uint64_t capacity, uint32_t b, uint64_t po) {
    if (b < 2 || b > 8 || (po & 3u) || po > capacity) return false;
    return payload_row_bytes(hidden, b) <= capacity - po;
}

// The CSR slice [rp0, rp1) of a token as restore reads it: ordered and inside the side stream.
TSQ_HD bool csr_slice_ok(uint64_t rp0, uint64_t rp1, uint64_t capacity) { return rp0 <= rp1 && rp1 <= capacity; }

// The CSR slice of a token as compress writes it: it must also hold exactly the token's `cnt` outliers.
TSQ_HD bool csr_slice_holds(uint64_t rp0, uint64_t rp1, uint64_t capacity, uint32_t cnt) {
    return csr_slice_ok(rp0, rp1, capacity) && rp1 - rp0 == (uint64_t)cnt;
}

// A column index read from the side stream.
TSQ_HD bool column_ok(uint32_t col, uint32_t hidden) { return col < hidden; }

// The stream [a, b) of one token inside the streams section of an entropy-coded blob: ordered, 4-byte
// aligned, inside the section, at least the `coders` 32-bit states long and no longer than a slot.
TSQ_HD bool stream_span_ok(uint64_t a, uint64_t b, uint64_t capacity, uint32_t coders, uint32_t slot_bytes) {
    if (a > b || b > capacity || (a & 3u)) return false;
    const uint64_t n = b - a;
    return n >= 4ull * coders && n <= (uint64_t)slot_bytes;
}

// A coded stream of `bytes` bytes moving from its slot to byte `at` of the streams section.
TSQ_HD bool stream_move_ok(uint32_t bytes, uint32_t coders, uint32_t slot_bytes, uint64_t at, uint64_t capacity) {
    if (bytes < 4u * coders || bytes > slot_bytes || at > capacity) return false;
    return (uint64_t)((bytes + 3u) & ~3u) <= capacity - at;
}

// Index into the 4096-entry cumulative-frequency table from a coder state.
TSQ_HD uint32_t frequency_slot(uint32_t state) { return state & 4095u; }

// The entropy coder's division.  floor(x / f) or one less, for x < f << 20 (so the quotient is below 2^20)
// and 1 <= f <= 4096, from `below` = the binary32 quotient 1 / f times (1 - 2^-21), rounded.  With e = 2^-24
// the unit roundoff: below lies in [(1 - 2^-21)(1 - e)^2 / f, (1 - 2^-21)(1 + e)^2 / f], and the product of
// (float)x and below carries two more roundings, so it lies in [x/f * (1 - 2^-21)(1 - e)^4,
// x/f * (1 - 2^-21)(1 + e)^4]: never above x/f (4e < 2^-21), and less than x/f * 12e < 0.75 below it.  Its
// integer part is therefore floor(x/f) or floor(x/f) - 1, which the size of the remainder tells.
TSQ_HD float reciprocal_just_below(uint32_t f) { return (1.0f / (float)f) * 0.999999523162841796875f; }   // 1 - 2^-21
TSQ_HD uint32_t quotient_or_one_less(uint32_t x, float below) { return (uint32_t)((float)x * below); }

// A workspace's recorded shape against the plan's.
TSQ_HD bool workspace_shape_ok(uint32_t ws_tokens, uint32_t ws_hidden, uint32_t tokens, uint32_t hidden) {
    return ws_tokens == tokens && ws_hidden == hidden;
}

}  // namespace tsq
