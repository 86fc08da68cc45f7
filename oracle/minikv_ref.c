/*
 * CPU oracle (test infrastructure, not the product) -- see minikv_ref.h for the contract.
 *
 * Written from the paper: the quantizer of Section 3.1.1 / Section 3.3 (asymmetric 2-bit, K grouped
 * along tokens per channel, V grouped along channels per token, 16 codes per 32-bit word, fp16 scale
 * and zero-point), the streaming residual buffer of Algorithm 1 lines 9-15, and the decode attention
 * of Algorithm 1 lines 17-19 with the 1/sqrt(d) of Appendix A eq. (1) supplied by the caller.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math: the code decisions
 * are defined by individually rounded IEEE binary32 operations).
 * The only parallelism is an OpenMP "for" over independent (batch, head) units.
 */
#include "minikv_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ fp16 conversions (bit level) */

float ref_f16_to_f32(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                  /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + m), e - 25);      /* (1 + m/1024) * 2^(e-15) */
    return (float)(sign ? -v : v);                   /* every binary16 is exact in binary32 */
}

/* Round a finite double to binary16, nearest-even, directly (no intermediate binary32). */
uint16_t ref_f64_to_f16(double x)
{
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000 : 0);
    double a = fabs(x);
    if (isnan(a)) return (uint16_t)(sign | 0x7e00);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7c00);
    int ex;
    (void)frexp(a, &ex);                             /* a = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;                                  /* a in [2^e, 2^(e+1)) */
    if (e < -14) {                                   /* subnormal range: units of 2^-24 */
        double q = nearbyint(ldexp(a, 24));          /* default rounding mode = nearest-even */
        return (uint16_t)(sign | (uint16_t)q);       /* q == 1024 lands on the smallest normal */
    }
    double m = nearbyint(ldexp(a, 10 - e));          /* in [1024, 2048] */
    if (m >= 2048.0) { m = 1024.0; e += 1; }
    if (e > 15) return (uint16_t)(sign | 0x7c00);
    return (uint16_t)(sign | ((e + 15) << 10) | ((int)m - 1024));
}

uint16_t ref_f32_to_f16(float f)
{
    return ref_f64_to_f16((double)f);                /* one rounding: binary32 is exact in binary64 */
}

/* ------------------------------------------------------------------ shapes and storage order */

int ref_check_shape(const ref_shape *s)
{
    if (!s) return -1;
    if (s->D != 128) return -1;
    if (!(s->G == 16 || s->G == 32 || s->G == 64 || s->G == 128)) return -1;
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv) return -1;
    if (s->Tcap <= 0 || s->Tcap % 128) return -1;
    if (s->Rcap < 0 || s->Rcap % s->G) return -1;
    return 0;
}

size_t ref_group_bytes(int G)
{
    return (size_t)G * 2 / 8 + 2 + 2;                /* G two-bit codes + fp16 scale + fp16 zero */
}

/* word index (within one unit's K code array) and bit position of token t, channel c */
static size_t k_slot(int t, int c, int *bit)
{
    int tile = t / 128, tau = t % 128;
    int w = c / 16;                                  /* which of the token's 8 words */
    *bit = 16 * (c % 2) + 2 * ((c % 16) / 2);
    return (size_t)tile * 1024 + (size_t)((2 * (tau % 2) + w / 4) * 64 + tau / 2) * 4 + (size_t)(w % 4);
}

/* word index (within one unit's V code array) and bit position of token t, channel c */
static size_t v_slot(int D, int t, int c, int *bit)
{
    int tile = t / 64, tau = t % 64;
    *bit = 16 * (tau % 2) + 2 * ((tau % 16) / 2);
    return (size_t)tile * 4 * (size_t)D + (size_t)c * 4 + (size_t)(tau / 16);
}

/* position of channel c inside a K scale / zero row: the 32 channel quads are dealt round-robin into
 * NB = G/8 bins, bin after bin */
int ref_k_meta_pos(int G, int c)
{
    int nb = G / 8, q = c / 4;
    return ((q % nb) * (32 / nb) + q / nb) * 4 + c % 4;
}

static size_t kc_words(const ref_shape *s) { return (size_t)s->Tcap / 128 * 1024; }
static size_t vc_words(const ref_shape *s) { return (size_t)s->Tcap / 64 * 4 * (size_t)s->D; }

/* ------------------------------------------------------------------ the 2-bit asymmetric quantizer */

/* zero-point = group minimum (stored in fp16, exact); scale = (max - min) / 3 rounded to fp16.
 * A zero of either sign is stored as +0. */
static void group_params(float mn, float mx, uint16_t *scale_h, uint16_t *zero_h, float *inv)
{
    uint16_t z = ref_f32_to_f16(mn);
    if ((z & 0x7fff) == 0) z = 0;
    float range = mx - mn;
    float step = range / 3.0f;
    uint16_t sh = ref_f32_to_f16(step);
    float sf = ref_f16_to_f32(sh);                   /* the STORED scale defines the codes */
    *scale_h = sh;
    *zero_h = z;
    *inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
}

/* code = clamp(round_half_even((x - zero) * (1/scale)), 0, 3); scale == 0 gives code 0 */
static int quant_code(float x, float zero, float inv)
{
    volatile float d = x - zero;                     /* volatile: two separately rounded binary32 ops */
    volatile float u = d * inv;
    float r = rintf(u);
    if (r < 0.0f) r = 0.0f;
    if (r > 3.0f) r = 3.0f;
    return (int)r;
}

/* Quantize and append n tokens (rows row[0..n-1] of Ksrc/Vsrc, each D fp16) to unit u at offset t0. */
static void quantize_unit(const ref_shape *s, ref_cache *c, size_t u, const uint16_t *Ksrc,
                          const uint16_t *Vsrc, const int32_t *row, int n, int t0)
{
    const int D = s->D, G = s->G;
    uint32_t *Kc = c->Kc + u * kc_words(s);
    uint32_t *Vc = c->Vc + u * vc_words(s);
    uint16_t *Ks = c->Ks + u * (size_t)(s->Tcap / G) * D;
    uint16_t *Kz = c->Kz + u * (size_t)(s->Tcap / G) * D;
    uint16_t *Vs = c->Vs + u * (size_t)s->Tcap * (D / G);
    uint16_t *Vz = c->Vz + u * (size_t)s->Tcap * (D / G);

    /* every word touched by the new tokens is rebuilt from zero (appends are whole words:
     * t0 and n are multiples of G >= 16) */
    for (int i = 0; i < n; i++) {
        int t = t0 + i, bit;
        for (int ch = 0; ch < D; ch += 16) Kc[k_slot(t, ch, &bit)] = 0;
        if (t % 16 == 0)
            for (int ch = 0; ch < D; ch++) Vc[v_slot(D, t, ch, &bit)] = 0;
    }

    /* K: per channel, groups of G consecutive retained tokens share (scale, zero) */
    for (int g0 = 0; g0 < n; g0 += G) {
        for (int ch = 0; ch < D; ch++) {
            float mn = INFINITY, mx = -INFINITY;
            for (int i = g0; i < g0 + G; i++) {
                float x = ref_f16_to_f32(Ksrc[(size_t)row[i] * D + ch]);
                if (x < mn) mn = x;
                if (x > mx) mx = x;
            }
            uint16_t sh, zh; float inv;
            group_params(mn, mx, &sh, &zh, &inv);
            size_t gidx = (size_t)((t0 + g0) / G) * D + ref_k_meta_pos(G, ch);
            Ks[gidx] = sh;
            Kz[gidx] = zh;
            float zf = ref_f16_to_f32(zh);
            for (int i = g0; i < g0 + G; i++) {
                float x = ref_f16_to_f32(Ksrc[(size_t)row[i] * D + ch]);
                int bit;
                size_t w = k_slot(t0 + i, ch, &bit);
                Kc[w] |= (uint32_t)quant_code(x, zf, inv) << bit;
            }
        }
    }

    /* V: per token, groups of G consecutive channels share (scale, zero) */
    for (int i = 0; i < n; i++) {
        for (int cg = 0; cg < D / G; cg++) {
            float mn = INFINITY, mx = -INFINITY;
            for (int ch = cg * G; ch < (cg + 1) * G; ch++) {
                float x = ref_f16_to_f32(Vsrc[(size_t)row[i] * D + ch]);
                if (x < mn) mn = x;
                if (x > mx) mx = x;
            }
            uint16_t sh, zh; float inv;
            group_params(mn, mx, &sh, &zh, &inv);
            size_t gidx = (size_t)(t0 + i) * (D / G) + cg;
            Vs[gidx] = sh;
            Vz[gidx] = zh;
            float zf = ref_f16_to_f32(zh);
            for (int ch = cg * G; ch < (cg + 1) * G; ch++) {
                float x = ref_f16_to_f32(Vsrc[(size_t)row[i] * D + ch]);
                int bit;
                size_t w = v_slot(D, t0 + i, ch, &bit);
                Vc[w] |= (uint32_t)quant_code(x, zf, inv) << bit;
            }
        }
    }
}

int kv_quantize_pack_ref(const ref_shape *s, const uint16_t *K, const uint16_t *V, int64_t L,
                         const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, ref_cache *c)
{
    if (ref_check_shape(s) || !K || !V || !n_tok || !c || L < 0) return -1;
    const size_t U = (size_t)s->B * s->Hkv;
    for (size_t u = 0; u < U; u++) {                 /* validate first, touch nothing on error */
        int n = n_tok[u], t0 = c->q_len[u];
        if (n < 0 || n % s->G || t0 < 0 || t0 % s->G || t0 + n > s->Tcap || n > L) return -1;
        if (idx) {
            if (n > idx_stride) return -1;
            for (int i = 0; i < n; i++) {
                int r = idx[u * (size_t)idx_stride + i];
                if (r < 0 || r >= L) return -1;
                if (i && r <= idx[u * (size_t)idx_stride + i - 1]) return -1;   /* ascending */
            }
        }
    }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (size_t u = 0; u < U; u++) {
        int n = n_tok[u];
        if (n == 0) continue;
        int32_t *row = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
        if (!row) { fail = 1; continue; }
        for (int i = 0; i < n; i++) row[i] = idx ? idx[u * (size_t)idx_stride + i] : i;
        quantize_unit(s, c, u, K + u * (size_t)L * s->D, V + u * (size_t)L * s->D, row, n, c->q_len[u]);
        c->q_len[u] += n;
        free(row);
    }
    return fail ? -1 : 0;
}

/* ------------------------------------------------------------------ residual buffer (Alg. 1, 9-15) */

int kv_append_residual_ref(const ref_shape *s, const uint16_t *k_new, const uint16_t *v_new, ref_cache *c)
{
    if (ref_check_shape(s) || !k_new || !v_new || !c) return -1;
    const size_t U = (size_t)s->B * s->Hkv;
    const int D = s->D;
    for (size_t u = 0; u < U; u++) {
        int r = c->r_len[u];
        if (r < 0 || r >= s->Rcap) continue;         /* full (or corrupt) unit: unchanged */
        memcpy(c->Rk + (u * (size_t)s->Rcap + r) * D, k_new + u * D, sizeof(uint16_t) * D);
        memcpy(c->Rv + (u * (size_t)s->Rcap + r) * D, v_new + u * D, sizeof(uint16_t) * D);
        c->r_len[u] = r + 1;
    }
    return 0;
}

int kv_flush_residual_ref(const ref_shape *s, ref_cache *c)
{
    if (ref_check_shape(s) || !c) return -1;
    const size_t U = (size_t)s->B * s->Hkv;
    const int D = s->D, R = s->Rcap;
    if (R == 0) return 0;
    int32_t *row = (int32_t *)malloc(sizeof(int32_t) * (size_t)R);
    if (!row) return -1;
    for (int i = 0; i < R; i++) row[i] = i;
    for (size_t u = 0; u < U; u++) {
        if (c->r_len[u] != R) continue;
        if (c->q_len[u] + R > s->Tcap) continue;     /* no room: left in the residual */
        quantize_unit(s, c, u, c->Rk + u * (size_t)R * D, c->Rv + u * (size_t)R * D, row, R, c->q_len[u]);
        c->q_len[u] += R;
        c->r_len[u] = 0;
    }
    free(row);
    return 0;
}

/* ------------------------------------------------------------------ layout-free views */

int ref_unpack_codes(const ref_shape *s, const ref_cache *c, int unit, uint8_t *Kcodes, uint8_t *Vcodes)
{
    if (ref_check_shape(s) || !c) return -1;
    const int D = s->D;
    const uint32_t *Kc = c->Kc + (size_t)unit * kc_words(s);
    const uint32_t *Vc = c->Vc + (size_t)unit * vc_words(s);
    int T = c->q_len[unit];
    for (int t = 0; t < T; t++)
        for (int ch = 0; ch < D; ch++) {
            int bit;
            size_t w = k_slot(t, ch, &bit);
            if (Kcodes) Kcodes[(size_t)t * D + ch] = (uint8_t)((Kc[w] >> bit) & 3u);
            w = v_slot(D, t, ch, &bit);
            if (Vcodes) Vcodes[(size_t)t * D + ch] = (uint8_t)((Vc[w] >> bit) & 3u);
        }
    return 0;
}

/* x_hat = code * scale + zero with the stored fp16 scale and zero, evaluated in binary64 (exact) */
int ref_dequant(const ref_shape *s, const ref_cache *c, int unit, double *Khat, double *Vhat)
{
    if (ref_check_shape(s) || !c) return -1;
    const int D = s->D, G = s->G;
    int T = c->q_len[unit];
    uint8_t *kc = (uint8_t *)malloc((size_t)(T ? T : 1) * D);
    uint8_t *vc = (uint8_t *)malloc((size_t)(T ? T : 1) * D);
    if (!kc || !vc) { free(kc); free(vc); return -1; }
    ref_unpack_codes(s, c, unit, kc, vc);
    const uint16_t *Ks = c->Ks + (size_t)unit * (s->Tcap / G) * D;
    const uint16_t *Kz = c->Kz + (size_t)unit * (s->Tcap / G) * D;
    const uint16_t *Vs = c->Vs + (size_t)unit * s->Tcap * (D / G);
    const uint16_t *Vz = c->Vz + (size_t)unit * s->Tcap * (D / G);
    for (int t = 0; t < T; t++)
        for (int ch = 0; ch < D; ch++) {
            size_t kg = (size_t)(t / G) * D + ref_k_meta_pos(G, ch);
            size_t vg = (size_t)t * (D / G) + ch / G;
            if (Khat) Khat[(size_t)t * D + ch] =
                (double)kc[(size_t)t * D + ch] * (double)ref_f16_to_f32(Ks[kg]) + (double)ref_f16_to_f32(Kz[kg]);
            if (Vhat) Vhat[(size_t)t * D + ch] =
                (double)vc[(size_t)t * D + ch] * (double)ref_f16_to_f32(Vs[vg]) + (double)ref_f16_to_f32(Vz[vg]);
        }
    free(kc); free(vc);
    return 0;
}

/* ------------------------------------------------------------------ decode attention (Alg. 1, 17-19) */

int minikv_decode_attn_ref(const ref_shape *s, const uint16_t *q, const ref_cache *c, float sm_scale,
                           uint16_t *out_f16, double *out_f64, double *probs)
{
    if (ref_check_shape(s) || !q || !c) return -1;
    const int D = s->D, G = s->G, Hq = s->Hq, Hkv = s->Hkv, R = s->Rcap;
    const int rep = Hq / Hkv;                        /* query heads sharing one KV head */
    const long NQ = (long)s->B * Hq;
    int fail = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (long bq = 0; bq < NQ; bq++) {
        int b = (int)(bq / Hq), hq = (int)(bq % Hq);
        size_t u = (size_t)b * Hkv + (size_t)(hq / rep);
        int T = c->q_len[u], r = c->r_len[u];
        if (T < 0) T = 0;
        if (T > s->Tcap) T = s->Tcap;
        if (r < 0) r = 0;
        if (r > R) r = R;
        int N = T + r;

        const uint32_t *Kc = c->Kc + u * kc_words(s);
        const uint32_t *Vc = c->Vc + u * vc_words(s);
        const uint16_t *Ks = c->Ks + u * (size_t)(s->Tcap / G) * D;
        const uint16_t *Kz = c->Kz + u * (size_t)(s->Tcap / G) * D;
        const uint16_t *Vs = c->Vs + u * (size_t)s->Tcap * (D / G);
        const uint16_t *Vz = c->Vz + u * (size_t)s->Tcap * (D / G);
        const uint16_t *Rk = c->Rk + u * (size_t)R * D;
        const uint16_t *Rv = c->Rv + u * (size_t)R * D;

        double qd[128], o[128];
        for (int ch = 0; ch < D; ch++) qd[ch] = (double)ref_f16_to_f32(q[(size_t)bq * D + ch]);
        for (int ch = 0; ch < D; ch++) o[ch] = 0.0;

        double *a = (double *)malloc(sizeof(double) * (size_t)(N ? N : 1));
        if (!a) { fail = 1; continue; }

        /* line 17: scores of the dequantized keys, then of the fp16 residual keys, one list */
        for (int t = 0; t < T; t++) {
            double acc = 0.0;
            for (int ch = 0; ch < D; ch++) {
                int bit;
                size_t w = k_slot(t, ch, &bit);
                double code = (double)((Kc[w] >> bit) & 3u);
                size_t g = (size_t)(t / G) * D + ref_k_meta_pos(G, ch);
                double khat = code * (double)ref_f16_to_f32(Ks[g]) + (double)ref_f16_to_f32(Kz[g]);
                acc += qd[ch] * khat;
            }
            a[t] = (double)sm_scale * acc;
        }
        for (int i = 0; i < r; i++) {
            double acc = 0.0;
            for (int ch = 0; ch < D; ch++) acc += qd[ch] * (double)ref_f16_to_f32(Rk[(size_t)i * D + ch]);
            a[T + i] = (double)sm_scale * acc;
        }

        /* one softmax over the concatenated scores */
        double mx = -INFINITY, sum = 0.0;
        for (int t = 0; t < N; t++) if (a[t] > mx) mx = a[t];
        for (int t = 0; t < N; t++) { a[t] = exp(a[t] - mx); sum += a[t]; }
        for (int t = 0; t < N; t++) a[t] /= sum;

        /* lines 18-19: A_quant * dequant(Q_V) + A_unquant * R_V */
        for (int t = 0; t < T; t++)
            for (int ch = 0; ch < D; ch++) {
                int bit;
                size_t w = v_slot(D, t, ch, &bit);
                double code = (double)((Vc[w] >> bit) & 3u);
                size_t g = (size_t)t * (D / G) + ch / G;
                double vhat = code * (double)ref_f16_to_f32(Vs[g]) + (double)ref_f16_to_f32(Vz[g]);
                o[ch] += a[t] * vhat;
            }
        for (int i = 0; i < r; i++)
            for (int ch = 0; ch < D; ch++)
                o[ch] += a[T + i] * (double)ref_f16_to_f32(Rv[(size_t)i * D + ch]);

        for (int ch = 0; ch < D; ch++) {
            if (out_f64) out_f64[(size_t)bq * D + ch] = o[ch];
            if (out_f16) out_f16[(size_t)bq * D + ch] = ref_f64_to_f16(o[ch]);
        }
        if (probs) {
            double *p = probs + (size_t)bq * (size_t)(s->Tcap + R);
            for (int t = 0; t < s->Tcap + R; t++) p[t] = 0.0;
            for (int t = 0; t < N; t++) p[t] = a[t];
        }
        free(a);
    }
    return fail ? -1 : 0;
}

/* ---------------------------------------------------------------------------------------------------
 * Token selection: Section 3.1.2 and Algorithm 1 line 3 (heavy hitters from the cumulative attention
 * score, plus the recent window).
 * ------------------------------------------------------------------------------------------------- */
typedef struct {
    float score;
    int32_t pos;
} scored_pos;

/* larger score first; of equal scores the earlier position first */
static int by_score_then_pos(const void *a, const void *b)
{
    const scored_pos *x = (const scored_pos *)a, *y = (const scored_pos *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int by_pos(const void *a, const void *b)
{
    const scored_pos *x = (const scored_pos *)a, *y = (const scored_pos *)b;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

int kv_select_hh_rw_ref(int32_t units, int32_t rep, int64_t L, const float *A_cumul,
                        const int32_t *n_hh, const int32_t *n_rw, int32_t *idx, int64_t idx_stride,
                        int32_t *n_tok)
{
    if (units < 0 || rep < 1 || L < 0 || L > INT32_MAX || idx_stride < 0) return -1;
    if (units > 0 && (!A_cumul || !n_hh || !n_rw || !idx || !n_tok)) return -1;
    scored_pos *cand = (scored_pos *)malloc(sizeof(scored_pos) * (size_t)(L > 0 ? L : 1));
    if (!cand) return -1;
    for (int32_t u = 0; u < units; ++u) {
        const int64_t rw = n_rw[u], hh = n_hh[u];
        if (rw < 0 || hh < 0 || rw > L || hh > L - rw || hh + rw > idx_stride) {
            n_tok[u] = 0;
            continue;
        }
        const int64_t n_cand = L - rw;                 /* the recent window is kept whatever its score */
        for (int64_t i = 0; i < n_cand; ++i) {
            float s = A_cumul[((size_t)u * (size_t)rep) * (size_t)L + (size_t)i];
            for (int32_t h = 1; h < rep; ++h)
                s = s + A_cumul[((size_t)u * (size_t)rep + (size_t)h) * (size_t)L + (size_t)i];
            cand[i].score = s;
            cand[i].pos = (int32_t)i;
        }
        qsort(cand, (size_t)n_cand, sizeof(scored_pos), by_score_then_pos);
        qsort(cand, (size_t)hh, sizeof(scored_pos), by_pos);      /* the heavy hitters, by position */
        int32_t *row = idx + (size_t)u * (size_t)idx_stride;
        for (int64_t i = 0; i < hh; ++i) row[i] = cand[i].pos;
        for (int64_t i = 0; i < rw; ++i) row[hh + i] = (int32_t)(n_cand + i);
        n_tok[u] = (int32_t)(hh + rw);
    }
    free(cand);
    return 0;
}

/* Section 3.1.3 (pyramid-like allocation) and the appendix paragraph on its details. */
int kv_pyramid_budget_ref(int32_t n_layers, double x, int32_t d, int32_t bottom_heavy, double *budget)
{
    if (n_layers < 1 || d < 1 || !(x >= 0.0) || !budget) return -1;
    if (n_layers == 1) {
        budget[0] = x;
        return 0;
    }
    const double small = x / (double)d, large = 2.0 * x - x / (double)d;
    const double first = bottom_heavy ? large : small, last = bottom_heavy ? small : large;
    for (int32_t l = 0; l < n_layers; ++l)
        budget[l] = first + (last - first) * (double)l / (double)(n_layers - 1);
    return 0;
}

/* ---------------------------------------------------------------------------------------------------
 * Prefill attention with cumulative attention scores: Section 3.2, Algorithm 1 line 2, eq. (1) (causal).
 * ------------------------------------------------------------------------------------------------- */
int selective_flash_attn_ref(int32_t B, int32_t Hq, int32_t Hkv, int64_t L, int32_t D, const uint16_t *Q,
                             const uint16_t *K, const uint16_t *V, float sm_scale, uint16_t *XO_f16,
                             double *XO_f64, double *lse, double *A_cumul)
{
    if (B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || L < 0 || D < 1 || !Q || !K || !V) return -1;
    const int rep = Hq / Hkv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < (long)B * Hq; ++bh) {
        const long b = bh / Hq, hq = bh % Hq, hk = hq / rep;
        const uint16_t *q = Q + (size_t)bh * (size_t)L * (size_t)D;
        const uint16_t *k = K + ((size_t)b * Hkv + (size_t)hk) * (size_t)L * (size_t)D;
        const uint16_t *v = V + ((size_t)b * Hkv + (size_t)hk) * (size_t)L * (size_t)D;
        double *p = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)D);
        if (!p || !o) {
            failed = 1;
            free(p);
            free(o);
            continue;
        }
        if (A_cumul)
            for (int64_t j = 0; j < L; ++j) A_cumul[(size_t)bh * (size_t)L + (size_t)j] = 0.0;
        for (int64_t i = 0; i < L; ++i) {
            double m = -INFINITY;
            for (int64_t j = 0; j <= i; ++j) {                 /* causal: keys up to the query's own position */
                double s = 0.0;
                for (int c = 0; c < D; ++c)
                    s += (double)ref_f16_to_f32(q[i * D + c]) * (double)ref_f16_to_f32(k[j * D + c]);
                p[j] = s * (double)sm_scale;
                if (p[j] > m) m = p[j];
            }
            double sum = 0.0;
            for (int64_t j = 0; j <= i; ++j) {
                p[j] = exp(p[j] - m);
                sum += p[j];
            }
            for (int c = 0; c < D; ++c) o[c] = 0.0;
            for (int64_t j = 0; j <= i; ++j) {
                p[j] /= sum;
                for (int c = 0; c < D; ++c) o[c] += p[j] * (double)ref_f16_to_f32(v[j * D + c]);
                if (A_cumul) A_cumul[(size_t)bh * (size_t)L + (size_t)j] += p[j];
            }
            const size_t row = ((size_t)bh * (size_t)L + (size_t)i);
            if (lse) lse[row] = m + log(sum);
            for (int c = 0; c < D; ++c) {
                if (XO_f64) XO_f64[row * (size_t)D + (size_t)c] = o[c];
                if (XO_f16) XO_f16[row * (size_t)D + (size_t)c] = ref_f64_to_f16(o[c]);
            }
        }
        free(p);
        free(o);
    }
    return failed ? -1 : 0;
}

/* The same attention for a list of query rows of ONE head (eq. (1), causal): what a full-size check can afford.
 * rows[r] in [0, L).  xo [n_rows][D], lse [n_rows]; p_tail [n_rows][tail] receives the row's weights of the LAST
 * `tail` keys (P[row][L - tail + t], zero for keys after the row), from which the caller can add up the
 * cumulative score of a late column over all the rows that see it.  Any output may be NULL. */
int selective_flash_attn_rows_ref(int64_t L, int32_t D, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                                  float sm_scale, const int64_t *rows, int32_t n_rows, double *xo, double *lse,
                                  double *p_tail, int32_t tail)
{
    if (L < 1 || D < 1 || !Q || !K || !V || !rows || n_rows < 0 || tail < 0 || tail > L) return -1;
    for (int r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= L) return -1;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        const int64_t i = rows[r];
        double *p = (double *)malloc(sizeof(double) * (size_t)(i + 1));
        if (!p) { failed = 1; continue; }
        double m = -INFINITY, sum = 0.0;
        for (int64_t j = 0; j <= i; ++j) {
            double s = 0.0;
            for (int c = 0; c < D; ++c)
                s += (double)ref_f16_to_f32(Q[i * D + c]) * (double)ref_f16_to_f32(K[j * D + c]);
            p[j] = s * (double)sm_scale;
            if (p[j] > m) m = p[j];
        }
        for (int64_t j = 0; j <= i; ++j) { p[j] = exp(p[j] - m); sum += p[j]; }
        for (int64_t j = 0; j <= i; ++j) p[j] /= sum;
        if (lse) lse[r] = m + log(sum);
        if (xo)
            for (int c = 0; c < D; ++c) {
                double o = 0.0;
                for (int64_t j = 0; j <= i; ++j) o += p[j] * (double)ref_f16_to_f32(V[j * D + c]);
                xo[(size_t)r * (size_t)D + (size_t)c] = o;
            }
        if (p_tail)
            for (int t = 0; t < tail; ++t) {
                const int64_t j = L - tail + t;
                p_tail[(size_t)r * (size_t)tail + (size_t)t] = j <= i ? p[j] : 0.0;
            }
        free(p);
    }
    return failed ? -1 : 0;
}
