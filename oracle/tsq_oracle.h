/*
 * tsq_oracle.h — plain CPU oracle for threshold splitting (TS) + token-wise
 * adaptive bit quantization (TAB-Q) and the exact inverse.
 *
 * TEST INFRASTRUCTURE ONLY.  This code exists to check the GPU library; it is
 * slow on purpose (scalar loops, no blocking, no fusion), shares no code with
 * the GPU path, and must never be called from it.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may use it.
 *
 * What it follows (paper: "Memory- and Latency-Constrained Inference of LLMs
 * via Adaptive Split Computing", Sec. II-C):
 *   - threshold splitting                : Eq. (ts)        (Sec. II-C.1)
 *   - CSR storage of the outlier part    : Sec. II-C.1, text after Eq. (ts)
 *   - integer quantization of magnitudes : Eq. (Proposed)  (Sec. II-C.2)
 *   - width descent with distortion test : Algorithm 1 (TAB-Q)
 *   - restore                            : Eq. (dequnt)
 *
 * Arithmetic contract: fp32 means IEEE binary32, round-to-nearest-even, no
 * fused multiply-add, no flush-to-zero; rint is round-half-to-even; integer
 * sums are exact; the per-token budget test is a fixed sequence of fp64
 * scalar operations.
 *
 * Pin status: every function here is pinned by tests/test_oracle_*.py against
 * closed forms, library routines (numpy / scipy / torch CPU), exact-rational
 * brute force and invariants.  The paper prints no worked numeric example of
 * TS, the quantizer or Algorithm 1, so against the paper's own numbers the
 * oracle is "parity unpinned".
 */
#ifndef TSQ_ORACLE_H
#define TSQ_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TSQO_F16  0
#define TSQO_BF16 1

#define TSQO_BUDGET_LSB     0   /* Algorithm 1's delta > Delta, in code LSBs        */
#define TSQO_BUDGET_REL_RMS 1   /* mean deviation vs budget * (row RMS), see .c    */

/* What Algorithm 1 returns when a candidate width exceeds the budget.  The steps as printed
 * quantize at the candidate, test, and on failure return THAT quantization ("break" comes after the
 * assignment of the result); the prose says the descent avoids excessive distortion, which fits the
 * last width that still passed.  LAST_PASSING is the reading the library defaults to; AS_PRINTED is
 * the printed order of steps.  If no candidate fails both give the smallest allowed width. */
#define TSQO_RETURN_LAST_PASSING 0
#define TSQO_RETURN_AS_PRINTED   1

/* Rows whose inlier absmax is below this are quantized as all-zero rows
 * (r = s = 0): below it Q_b/amax can overflow binary32. */
#define TSQO_AMAX_FLOOR 0x1p-100f

typedef struct {
    uint32_t tokens;     /* T >= 1                                           */
    uint32_t hidden;     /* H >= 1, H <= 65536 (CSR columns are u16)         */
    int32_t  dtype;      /* TSQO_F16 / TSQO_BF16                             */
    float    tau;        /* threshold, 0 < tau < inf                         */
    uint32_t bit_mask;   /* bit b set <=> width b allowed, 2 <= b <= 8       */
    float    budget;     /* Delta (LSB mode) or epsilon (REL_RMS mode), >= 0 */
    int32_t  mode;       /* TSQO_BUDGET_*                                    */
    int32_t  rule;       /* TSQO_RETURN_*: which width Algorithm 1 returns   */
} tsqo_config;

typedef struct {
    uint32_t cnt;        /* outliers in this token                            */
    float    amax;       /* max |x| over inliers (0 if none)                  */
    uint32_t bits;       /* chosen width b_t                                  */
    float    scale;      /* s_t = amax / Q_{b_t} (0 for an all-zero row)      */
    uint32_t nbytes;     /* payload bytes of the token = 4*ceil(H*b_t/32)     */
    uint32_t n_eval;     /* candidates whose statistic was evaluated          */
    uint64_t ss0;        /* sum of squared reference codes                    */
    uint64_t sad[8];     /* sad[i]: statistic of the i-th candidate (i>=1),
                            candidates in descending width order; 0 if not
                            evaluated                                         */
} tsqo_token_info;

/* 16-bit storage value -> binary32 (exact). */
float    tsqo_widen(uint16_t raw, int32_t dtype);
/* binary32 -> 16-bit storage value, round-to-nearest-even. */
uint16_t tsqo_narrow(float v, int32_t dtype);

/* Eq. (ts) on one token: out[j] = !(|x_j| < tau); a[j] = out ? 0 : |x_j|. */
void tsqo_ts_row(const uint16_t *x, uint32_t H, int32_t dtype, float tau,
                 uint8_t *out, float *a, uint32_t *cnt, float *amax);

/* Eq. (Proposed) on magnitudes with T_min = 0: r = Q_b/amax, s = amax/Q_b,
 * m[j] = min(rint(a[j]*r), Q_b).  b is the total width including the sign. */
void tsqo_aiq_row(const float *a, uint32_t H, float amax, int b,
                  int32_t *m, float *r, float *s);

/* Algorithm 1's descent over the allowed widths for one token (TSQO_RETURN_LAST_PASSING). */
void tsqo_select_row(const float *a, uint32_t H, float amax, uint32_t bit_mask,
                     float budget, int32_t mode, tsqo_token_info *info);
/* The same with the return rule chosen by the caller (TSQO_RETURN_*). */
void tsqo_select_row_rule(const float *a, uint32_t H, float amax, uint32_t bit_mask,
                          float budget, int32_t mode, int32_t rule, tsqo_token_info *info);

/* Dense LSB-first bit stream of b-bit sign|magnitude codes, zero padded to a
 * 4-byte multiple.  dst must hold 4*ceil(H*b/32) bytes. */
void tsqo_pack_row(const int32_t *m, const uint8_t *neg, uint32_t H, int b,
                   uint8_t *dst);
void tsqo_unpack_row(const uint8_t *src, uint32_t H, int b,
                     int32_t *m, uint8_t *neg);

/* Whole tensor.  Returns 0 on success, 1 on bad config, 3 if a capacity is too
 * small (then pay_off / row_ptr / bits / scale are still complete).
 * info may be NULL.  nthreads <= 1 runs serially. */
int tsqo_compress(const tsqo_config *cfg, const uint16_t *x,
                  uint8_t *bits, float *scale,
                  uint64_t *pay_off, uint64_t *row_ptr,
                  uint8_t *payload, uint64_t payload_cap,
                  uint16_t *out_col, uint16_t *out_val, uint64_t out_cap,
                  tsqo_token_info *info, int nthreads);

/* Eq. (dequnt).  Only tokens, hidden and dtype of cfg are used. */
int tsqo_decompress(const tsqo_config *cfg,
                    const uint8_t *bits, const float *scale,
                    const uint64_t *pay_off, const uint64_t *row_ptr,
                    const uint8_t *payload,
                    const uint16_t *out_col, const uint16_t *out_val,
                    uint16_t *out, int nthreads);

/* OpenMP threads available to the two calls above (1 if built without). */
int tsqo_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif
