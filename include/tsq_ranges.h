/*
 * tsq_ranges.h — the admissibility checks that the kernels apply to offsets, sizes and indices they
 * read from a blob, an entropy-coded blob or a workspace before using them as addresses, evaluated
 * on the HOST.  Each call runs the very predicate the kernels compile (one source, built for both
 * sides), so that a test without a GPU can drive it with wrapping offsets and noise.  Plain values
 * in, 1 (admissible) or 0 out; no device, no errors.  tsq_check_quotients does the same for the one step of
 * the entropy coder's arithmetic that rests on a rounding argument.
 */
#ifndef TSQ_RANGES_H
#define TSQ_RANGES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A token of `width` bits per element whose codes start at byte `offset` of a payload section of
 * `capacity` bytes: width in 2..8, offset 4-byte aligned, the 4*ceil(hidden*width/32) bytes inside. */
int tsq_check_payload_span(uint32_t hidden, uint64_t capacity, uint32_t width, uint64_t offset);
/* CSR slice [rp0, rp1) of a token as restore reads it: ordered, inside a side stream of `capacity` entries. */
int tsq_check_csr_slice(uint64_t rp0, uint64_t rp1, uint64_t capacity);
/* ... as compress writes it: it must also hold exactly `count` entries. */
int tsq_check_csr_slice_holds(uint64_t rp0, uint64_t rp1, uint64_t capacity, uint32_t count);
/* A column index from the side stream. */
int tsq_check_column(uint32_t column, uint32_t hidden);
/* Stream [begin, end) of a token in the streams section of an entropy-coded blob: ordered, 4-byte
 * aligned, inside `capacity`, at least 4*coders bytes (the coder states) and at most slot_bytes. */
int tsq_check_stream_span(uint64_t begin, uint64_t end, uint64_t capacity, uint32_t coders, uint32_t slot_bytes);
/* A coded stream of `bytes` bytes moving to byte `at` of the streams section (padded to 4 bytes). */
int tsq_check_stream_move(uint32_t bytes, uint32_t coders, uint32_t slot_bytes, uint64_t at, uint64_t capacity);
/* Index into the 4096-entry frequency table from a coder state (always below 4096). */
uint32_t tsq_check_frequency_slot(uint32_t state);
/* The entropy encoder's division step, for n pairs (HOST arrays): q[i] = the encoder's first estimate of
 * floor(x[i] / f[i]), which is that quotient or one less whenever 1 <= f[i] <= 4096 and x[i] < f[i] << 20
 * (the encoder then corrects it by the size of the remainder). */
void tsq_check_quotients(const uint32_t *x, const uint32_t *f, uint32_t *q, uint64_t n);
/* The shape recorded in a workspace against the plan's. */
int tsq_check_workspace_shape(uint32_t ws_tokens, uint32_t ws_hidden, uint32_t tokens, uint32_t hidden);

#ifdef __cplusplus
}
#endif
#endif /* TSQ_RANGES_H */
