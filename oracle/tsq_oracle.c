/*
 * tsq_oracle.c — plain CPU oracle for TS + TAB-Q (see tsq_oracle.h).
 *
 * TEST INFRASTRUCTURE ONLY: never part of the product path.
 *
 * The method is a lossy encoding chosen by a sequential heuristic, so this
 * file takes the algorithm's steps in the paper's order, one plain loop per
 * step, with no blocking, fusion or reordering.  Build with
 *   gcc -O2 -ffp-contract=off -fno-fast-math [-fopenmp]
 * so that every fp32 operation below is one IEEE operation.
 */
#include "tsq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* 16-bit storage formats                                              */
/* ------------------------------------------------------------------ */

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

float tsqo_widen(uint16_t raw, int32_t dtype)
{
    if (dtype == TSQO_BF16)                      /* bf16 = upper half of binary32 */
        return bits_to_float((uint32_t)raw << 16);

    /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
    uint32_t sign = (raw >> 15) & 1u;
    uint32_t e    = (raw >> 10) & 0x1Fu;
    uint32_t f    = raw & 0x3FFu;
    float mag;
    if (e == 0)        mag = ldexpf((float)f, -24);                 /* zero / subnormal */
    else if (e == 31)  mag = f ? bits_to_float(0x7F800000u | (f << 13)) /* NaN, payload kept */
                               : INFINITY;
    else               mag = ldexpf((float)(1024u + f), (int)e - 25);
    if (e == 31 && f)  return bits_to_float(float_to_bits(mag) | (sign << 31));
    return sign ? -mag : mag;
}

uint16_t tsqo_narrow(float v, int32_t dtype)
{
    uint32_t u = float_to_bits(v);
    uint32_t sign = u >> 31;
    uint32_t absu = u & 0x7FFFFFFFu;

    if (dtype == TSQO_BF16) {
        if (absu > 0x7F800000u)                  /* NaN: keep it a NaN */
            return (uint16_t)((u >> 16) | 0x0040u);
        /* keep 16 of 32 bits; ties go to the even 16-bit pattern */
        uint32_t keep = u >> 16, rest = u & 0xFFFFu;
        if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
        return (uint16_t)keep;                   /* carry into the exponent is correct, incl. -> inf */
    }

    /* binary16 */
    if (absu > 0x7F800000u) return (uint16_t)((sign << 15) | 0x7E00u);
    if (absu == 0x7F800000u) return (uint16_t)((sign << 15) | 0x7C00u);
    float a = fabsf(v);
    if (a == 0.0f) return (uint16_t)(sign << 15);
    int ex;
    (void)frexpf(a, &ex);                        /* a = frac * 2^ex, frac in [0.5,1) */
    int e = ex - 1;                              /* a in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;                        /* subnormal binary16: fixed spacing 2^-24 */
    /* spacing of binary16 at this exponent is 2^(e-10); a / spacing is exact in
       binary32 (power-of-two scaling, result < 2^12), rintf rounds half to even */
    float q = rintf(ldexpf(a, 10 - e));          /* in [0, 2048] */
    uint32_t qi = (uint32_t)q;
    uint32_t h;
    if (e == -14 && qi < 1024u) {
        h = qi;                                  /* subnormal (or zero) */
    } else {
        if (qi == 2048u) { qi = 1024u; e += 1; } /* rounded up to the next binade */
        if (e > 15) h = 0x7C00u;                 /* overflow -> inf */
        else        h = ((uint32_t)(e + 15) << 10) | (qi - 1024u);
    }
    return (uint16_t)((sign << 15) | h);
}

/* ------------------------------------------------------------------ */
/* Eq. (ts): threshold splitting of one token                          */
/* ------------------------------------------------------------------ */

void tsqo_ts_row(const uint16_t *x, uint32_t H, int32_t dtype, float tau,
                 uint8_t *out, float *a, uint32_t *cnt, float *amax)
{
    uint32_t c = 0;
    float mx = 0.0f;
    for (uint32_t j = 0; j < H; ++j) {
        float v  = tsqo_widen(x[j], dtype);
        float av = fabsf(v);
        /* M_ij = 1 iff |T_ij| >= tau.  Written as the negation of "<" so that
           NaN (which compares false) and +-Inf land on the lossless side. */
        int is_out = !(av < tau);
        out[j] = (uint8_t)is_out;
        a[j]   = is_out ? 0.0f : av;             /* |T_below|: zero at masked slots */
        c += (uint32_t)is_out;
        if (a[j] > mx) mx = a[j];
    }
    *cnt  = c;
    *amax = mx;
}

/* ------------------------------------------------------------------ */
/* Eq. (Proposed) on magnitudes, T_min = 0 so the zero point is 0      */
/* ------------------------------------------------------------------ */

void tsqo_aiq_row(const float *a, uint32_t H, float amax, int b,
                  int32_t *m, float *r, float *s)
{
    float Q = (float)((1 << (b - 1)) - 1);       /* Q_max = 2^(b-1) - 1 */
    float rr = 0.0f, ss = 0.0f;
    if (amax >= TSQO_AMAX_FLOOR) {
        rr = Q / amax;                           /* 1/s, rounded once */
        ss = amax / Q;                           /* s = (T_max - 0) / Q_max */
    }
    for (uint32_t j = 0; j < H; ++j) {
        float t = rintf(a[j] * rr);              /* round(T/s), half to even */
        if (t > Q) t = Q;
        m[j] = (int32_t)t;
    }
    *r = rr;
    *s = ss;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1: descend through the allowed widths                     */
/* ------------------------------------------------------------------ */

void tsqo_select_row(const float *a, uint32_t H, float amax, uint32_t bit_mask,
                     float budget, int32_t mode, tsqo_token_info *info)
{
    tsqo_select_row_rule(a, H, amax, bit_mask, budget, mode, TSQO_RETURN_LAST_PASSING, info);
}

void tsqo_select_row_rule(const float *a, uint32_t H, float amax, uint32_t bit_mask,
                          float budget, int32_t mode, int32_t rule, tsqo_token_info *info)
{
    int widths[8], k = 0;
    for (int b = 8; b >= 2; --b)                 /* allowed widths, descending */
        if (bit_mask & (1u << b)) widths[k++] = b;

    int32_t *m0 = (int32_t *)malloc(sizeof(int32_t) * (size_t)H);
    int32_t *mb = (int32_t *)malloc(sizeof(int32_t) * (size_t)H);
    float r, s;

    /* reference quantization at the largest width */
    int b0 = widths[0];
    tsqo_aiq_row(a, H, amax, b0, m0, &r, &s);
    uint64_t ss0 = 0;
    for (uint32_t j = 0; j < H; ++j) ss0 += (uint64_t)m0[j] * (uint64_t)m0[j];

    memset(info->sad, 0, sizeof info->sad);
    info->ss0    = ss0;
    info->n_eval = 0;
    int   sel    = b0;
    float sel_s  = s;
    double Q0 = (double)((1 << (b0 - 1)) - 1);

    for (int i = 1; i < k; ++i) {
        int bi = widths[i];
        tsqo_aiq_row(a, H, amax, bi, mb, &r, &s);
        /* delta * n = sum | floor(T0 / 2^(b0-bi)) - T | : an exact integer */
        uint64_t sad = 0;
        for (uint32_t j = 0; j < H; ++j) {
            int32_t d = (m0[j] >> (b0 - bi)) - mb[j];
            sad += (uint64_t)(d < 0 ? -d : d);
        }
        info->sad[i] = sad;
        info->n_eval = (uint32_t)i;

        int viol;
        if (mode == TSQO_BUDGET_LSB) {
            /* delta > Delta  <=>  sad > Delta * n */
            viol = (double)sad > (double)budget * (double)H;
        } else {
            /* mean value-domain deviation s_bi*sad/H against
               budget * RMS, RMS = s_b0 * sqrt(ss0/H); with s_bi/s_b0 = Q0/Qi
               this is (Q0*sad)^2 > (budget*Qi)^2 * H * ss0 */
            double Qi = (double)((1 << (bi - 1)) - 1);
            double L = Q0 * (double)sad;
            L *= L;
            double R = (double)budget * Qi;
            R *= R;
            R *= (double)H;
            R *= (double)ss0;
            viol = L > R;
        }
        if (viol && rule == TSQO_RETURN_LAST_PASSING)
            break;                               /* keep the last width that passed */
        sel   = bi;
        sel_s = s;
        if (viol) break;                         /* as printed: the failing width is what is returned */
    }

    info->amax   = amax;
    info->bits   = (uint32_t)sel;
    info->scale  = sel_s;
    info->nbytes = 4u * (uint32_t)(((uint64_t)H * (uint64_t)sel + 31u) / 32u);
    free(m0);
    free(mb);
}

/* ------------------------------------------------------------------ */
/* Bit stream of one token                                             */
/* ------------------------------------------------------------------ */

void tsqo_pack_row(const int32_t *m, const uint8_t *neg, uint32_t H, int b,
                   uint8_t *dst)
{
    uint64_t nbytes = 4u * (((uint64_t)H * (uint64_t)b + 31u) / 32u);
    memset(dst, 0, (size_t)nbytes);
    for (uint32_t j = 0; j < H; ++j) {
        uint32_t code = ((uint32_t)(neg[j] ? 1u : 0u) << (b - 1)) | (uint32_t)m[j];
        for (int k = 0; k < b; ++k) {            /* code bit k -> stream bit j*b + k */
            uint64_t i = (uint64_t)j * (uint64_t)b + (uint64_t)k;
            if ((code >> k) & 1u) dst[i >> 3] |= (uint8_t)(1u << (i & 7u));
        }
    }
}

void tsqo_unpack_row(const uint8_t *src, uint32_t H, int b,
                     int32_t *m, uint8_t *neg)
{
    for (uint32_t j = 0; j < H; ++j) {
        uint32_t code = 0;
        for (int k = 0; k < b; ++k) {
            uint64_t i = (uint64_t)j * (uint64_t)b + (uint64_t)k;
            code |= (uint32_t)((src[i >> 3] >> (i & 7u)) & 1u) << k;
        }
        neg[j] = (uint8_t)(code >> (b - 1));
        m[j]   = (int32_t)(code & ((1u << (b - 1)) - 1u));
    }
}

/* ------------------------------------------------------------------ */
/* Whole tensor                                                        */
/* ------------------------------------------------------------------ */

static int config_ok(const tsqo_config *c)
{
    if (!c || c->tokens == 0 || c->hidden == 0 || c->hidden > 65536u) return 0;
    if (c->dtype != TSQO_F16 && c->dtype != TSQO_BF16) return 0;
    if (!(c->tau > 0.0f) || isinf(c->tau)) return 0;
    if ((c->bit_mask & 0x1FCu) == 0 || (c->bit_mask & ~0x1FCu) != 0) return 0;
    if (!(c->budget >= 0.0f)) return 0;
    if (c->mode != TSQO_BUDGET_LSB && c->mode != TSQO_BUDGET_REL_RMS) return 0;
    return 1;
}

int tsqo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int tsqo_compress(const tsqo_config *cfg, const uint16_t *x,
                  uint8_t *bits, float *scale,
                  uint64_t *pay_off, uint64_t *row_ptr,
                  uint8_t *payload, uint64_t payload_cap,
                  uint16_t *out_col, uint16_t *out_val, uint64_t out_cap,
                  tsqo_token_info *info, int nthreads)
{
    if (!config_ok(cfg)) return 1;
    const uint32_t T = cfg->tokens, H = cfg->hidden;
    if (nthreads < 1) nthreads = 1;
    (void)nthreads;

    tsqo_token_info *ti = info ? info
                               : (tsqo_token_info *)malloc(sizeof(tsqo_token_info) * (size_t)T);

    /* per token: split, then choose the width */
    #pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t t = 0; t < (int64_t)T; ++t) {
        uint8_t *out = (uint8_t *)malloc(H);
        float   *a   = (float *)malloc(sizeof(float) * (size_t)H);
        uint32_t cnt; float amax;
        tsqo_ts_row(x + (size_t)t * H, H, cfg->dtype, cfg->tau, out, a, &cnt, &amax);
        tsqo_select_row_rule(a, H, amax, cfg->bit_mask, cfg->budget, cfg->mode, cfg->rule, &ti[t]);
        ti[t].cnt = cnt;
        bits[t]   = (uint8_t)ti[t].bits;
        scale[t]  = ti[t].scale;
        free(out); free(a);
    }

    /* CSR row pointers and payload offsets: exclusive running sums */
    row_ptr[0] = 0; pay_off[0] = 0;
    for (uint32_t t = 0; t < T; ++t) {
        row_ptr[t + 1] = row_ptr[t] + ti[t].cnt;
        pay_off[t + 1] = pay_off[t] + ti[t].nbytes;
    }
    int rc = 0;
    if (row_ptr[T] > out_cap || pay_off[T] > payload_cap) rc = 3;

    if (rc == 0) {
        #pragma omp parallel for schedule(static) num_threads(nthreads)
        for (int64_t t = 0; t < (int64_t)T; ++t) {
            const uint16_t *row = x + (size_t)t * H;
            uint8_t *out = (uint8_t *)malloc(H);
            uint8_t *neg = (uint8_t *)malloc(H);
            float   *a   = (float *)malloc(sizeof(float) * (size_t)H);
            int32_t *m   = (int32_t *)malloc(sizeof(int32_t) * (size_t)H);
            uint32_t cnt; float amax, r, s;
            tsqo_ts_row(row, H, cfg->dtype, cfg->tau, out, a, &cnt, &amax);

            /* T_above of this token, in CSR: ascending columns, raw values */
            uint64_t p = row_ptr[t];
            for (uint32_t j = 0; j < H; ++j)
                if (out[j]) { out_col[p] = (uint16_t)j; out_val[p] = row[j]; ++p; }

            /* T_below of this token at the chosen width; sign kept beside the
               magnitude, and dropped where the magnitude is zero */
            int b = (int)ti[t].bits;
            tsqo_aiq_row(a, H, amax, b, m, &r, &s);
            for (uint32_t j = 0; j < H; ++j) {
                int sign = (row[j] >> 15) & 1;
                neg[j] = (uint8_t)(sign && m[j] > 0 && !out[j]);
            }
            tsqo_pack_row(m, neg, H, b, payload + pay_off[t]);
            free(out); free(neg); free(a); free(m);
        }
    }
    if (!info) free(ti);
    return rc;
}

int tsqo_decompress(const tsqo_config *cfg,
                    const uint8_t *bits, const float *scale,
                    const uint64_t *pay_off, const uint64_t *row_ptr,
                    const uint8_t *payload,
                    const uint16_t *out_col, const uint16_t *out_val,
                    uint16_t *out, int nthreads)
{
    if (!cfg || cfg->tokens == 0 || cfg->hidden == 0) return 1;
    const uint32_t T = cfg->tokens, H = cfg->hidden;
    if (nthreads < 1) nthreads = 1;
    (void)nthreads;

    #pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t t = 0; t < (int64_t)T; ++t) {
        int32_t *m   = (int32_t *)malloc(sizeof(int32_t) * (size_t)H);
        uint8_t *neg = (uint8_t *)malloc(H);
        uint16_t *row = out + (size_t)t * H;
        int b = (int)bits[t];
        tsqo_unpack_row(payload + pay_off[t], H, b, m, neg);
        /* (T_hat - 0) * S, sign re-applied */
        for (uint32_t j = 0; j < H; ++j) {
            float v = (float)m[j] * scale[t];
            if (neg[j]) v = -v;
            row[j] = tsqo_narrow(v, cfg->dtype);
        }
        /* + T_above: outliers go back untouched */
        for (uint64_t p = row_ptr[t]; p < row_ptr[t + 1]; ++p)
            row[out_col[p]] = out_val[p];
        free(m); free(neg);
    }
    return 0;
}
