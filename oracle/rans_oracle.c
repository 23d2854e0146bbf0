/*
 * The token coder of rans_oracle.py once more in plain C, so that whole tensors can be coded in
 * seconds.  TEST INFRASTRUCTURE ONLY (see tsq_oracle.py): the format is the one stated at the top of
 * rans_oracle.py (rANS as published, 32-bit state, 16-bit words, 12-bit frequencies, 64 coders per
 * token over runs of 32 codes, the encoder walking the steps backwards).  One symbol at a time, no
 * blocking or reordering; tests pin it to the Python coder, which is pinned by hand-worked streams.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PROB_BITS 12
#define LOW (1u << 16)
#define CODERS 64u
#define RUN 32u

/* codes: H codes of one token; freq: the 256 frequencies of its width class; out: room for
 * 4 * 64 + 2 * H + 4 bytes.  Returns the stream's length in bytes (a multiple of 4). */
uint32_t ranso_encode_token(const uint8_t *codes, uint32_t H, const uint16_t *freq, uint8_t *out) {
    uint32_t cum[256], c = 0;
    for (int s = 0; s < 256; ++s) { cum[s] = c; c += freq[s]; }
    const uint32_t runs = (H + RUN - 1) / RUN;
    const uint32_t steps = RUN * ((runs + CODERS - 1) / CODERS);
    const uint32_t in_use = runs < CODERS ? runs : CODERS;
    uint32_t x[CODERS];
    for (uint32_t l = 0; l < CODERS; ++l) x[l] = LOW;
    /* the words of every step, in coder order */
    uint16_t *w = (uint16_t *)malloc((size_t)steps * CODERS * sizeof(uint16_t));
    uint32_t *n = (uint32_t *)calloc(steps, sizeof(uint32_t));
    if (!w || !n) { free(w); free(n); return 0; }
    for (uint32_t i = steps; i-- > 0;) {
        for (uint32_t l = 0; l < CODERS; ++l) {
            const uint64_t e = ((uint64_t)l + CODERS * (i / RUN)) * RUN + (i % RUN);
            if (e >= H) continue;
            const uint32_t s = codes[e], f = freq[s];
            if (f == 0) { free(w); free(n); return 0; }          /* a code that the table does not know */
            if ((uint64_t)x[l] >= ((uint64_t)f << 20)) {       /* f may be 4096: the bound is 2^32 then */
                w[(size_t)i * CODERS + n[i]++] = (uint16_t)(x[l] & 0xFFFFu);
                x[l] >>= 16;
            }
            x[l] = ((x[l] / f) << PROB_BITS) + (x[l] % f) + cum[s];
        }
    }
    uint32_t at = 0;
    for (uint32_t l = 0; l < in_use; ++l) { memcpy(out + at, &x[l], 4); at += 4; }
    for (uint32_t i = 0; i < steps; ++i)
        for (uint32_t k = 0; k < n[i]; ++k) { memcpy(out + at, &w[(size_t)i * CODERS + k], 2); at += 2; }
    while (at & 3u) out[at++] = 0;
    free(w);
    free(n);
    return at;
}

/* codes: T x H codes; bits: the tokens' widths; tables: 7 x 256 frequencies (row b - 2: width b).
 * off: T + 1 stream offsets out; streams: `capacity` bytes.  Returns the bytes used, or 0 if a
 * token could not be coded or the streams do not fit. */
uint64_t ranso_encode(const uint8_t *codes, const uint8_t *bits, const uint16_t *tables, uint32_t T, uint32_t H,
                      uint64_t *off, uint8_t *streams, uint64_t capacity) {
    const size_t slot = 4u * CODERS + 2u * (size_t)H + 4u;
    uint8_t *slots = (uint8_t *)malloc(slot * T);
    uint32_t *len = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)T);
    if (!slots || !len) { free(slots); free(len); return 0; }
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < (int64_t)T; ++t) {
        const uint32_t b = bits[t];
        len[t] = (b >= 2 && b <= 8) ? ranso_encode_token(codes + (size_t)t * H, H, tables + (size_t)(b - 2) * 256, slots + slot * (size_t)t) : 0;
        if (len[t] == 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    uint64_t at = 0;
    for (uint32_t t = 0; t < T && !bad; ++t) {
        off[t] = at;
        if (at + len[t] > capacity) { bad = 1; break; }
        memcpy(streams + at, slots + slot * (size_t)t, len[t]);
        at += len[t];
    }
    if (!bad) off[T] = at;
    free(slots);
    free(len);
    return bad ? 0 : at;
}
