/*
 * CPU oracle (test infrastructure, not the product), second part -- see minikv_pt_ref.h for the contract:
 * per-token asymmetric quantization of keys and values with 2, 4 or 8 bits (the token-wise quantization of
 * the paper's appendix and its 4-bit baseline) and attention over the dequantized cache (Appendix A eq. (1)).
 * Plain loops, fp64 sums, no blocking; OpenMP only across independent units / query rows.
 */
#include "minikv_pt_ref.h"
#include "minikv_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

int ref_pt_check_shape(const ref_pt_shape *s)
{
    if (!s) return -1;
    if (s->D != 128) return -1;
    if (!(s->G == 32 || s->G == 64 || s->G == 128)) return -1;
    if (!(s->bits == 2 || s->bits == 4 || s->bits == 8)) return -1;
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv) return -1;
    if (s->Tcap <= 0 || s->Tcap % 64) return -1;
    return 0;
}

size_t ref_pt_token_bytes(int D, int G, int bits)
{
    return (size_t)D * (size_t)bits / 8 + (size_t)(D / G) * 4;
}

/* where the code of (token t, channel ch) lives */
static size_t pt_k_slot(const ref_pt_shape *s, int t, int ch, int *bit)
{
    int cpw = 32 / s->bits;
    *bit = s->bits * (ch % cpw);
    return (size_t)t * (size_t)(s->D / cpw) + (size_t)(ch / cpw);
}
static size_t pt_v_slot(const ref_pt_shape *s, int t, int ch, int *bit)
{
    int cpw = 32 / s->bits;
    *bit = s->bits * (t % cpw);
    return (size_t)(t / cpw) * (size_t)s->D + (size_t)ch;
}
static size_t pt_kc_words(const ref_pt_shape *s) { return (size_t)s->Tcap * (size_t)(s->D * s->bits / 32); }
static size_t pt_vc_words(const ref_pt_shape *s) { return (size_t)(s->Tcap * s->bits / 32) * (size_t)s->D; }

/* zero-point, scale and reciprocal of one group with extrema mn, mx and `levels` = 2^bits - 1 steps */
static void pt_group_params(float mn, float mx, int levels, uint16_t *scale_h, uint16_t *zero_h, float *inv)
{
    uint16_t z = ref_f32_to_f16(mn);
    if ((z & 0x7fff) == 0) z = 0;
    float range = mx - mn;
    float step = range / (float)levels;
    uint16_t sh = ref_f32_to_f16(step);
    float sf = ref_f16_to_f32(sh);
    *scale_h = sh;
    *zero_h = z;
    *inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
}

static int pt_quant_code(float x, float zero, float inv, int levels)
{
    volatile float d = x - zero;                     /* two separately rounded binary32 operations */
    volatile float u = d * inv;
    float r = rintf(u);
    if (r < 0.0f) r = 0.0f;
    if (r > (float)levels) r = (float)levels;
    return (int)r;
}

/* one row (token) of one tensor: scales, zero-points and codes of its D/G groups */
static void pt_quantize_row(const ref_pt_shape *s, const uint16_t *row, uint16_t *sc, uint16_t *zp, int *codes)
{
    const int D = s->D, G = s->G, levels = (1 << s->bits) - 1;
    for (int g = 0; g < D / G; g++) {
        float mn = INFINITY, mx = -INFINITY;
        for (int ch = g * G; ch < (g + 1) * G; ch++) {
            float x = ref_f16_to_f32(row[ch]);
            if (x < mn) mn = x;
            if (x > mx) mx = x;
        }
        float inv;
        pt_group_params(mn, mx, levels, &sc[g], &zp[g], &inv);
        float zf = ref_f16_to_f32(zp[g]);
        for (int ch = g * G; ch < (g + 1) * G; ch++)
            codes[ch] = pt_quant_code(ref_f16_to_f32(row[ch]), zf, inv, levels);
    }
}

int kv_quantize_pack_pt_ref(const ref_pt_shape *s, const uint16_t *K, const uint16_t *V, int64_t L,
                            const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, ref_pt_cache *c)
{
    if (ref_pt_check_shape(s) || !K || !V || !n_tok || !c || L < 0) return -1;
    const size_t U = (size_t)s->B * s->Hkv;
    const int D = s->D, NG = s->D / s->G;
    for (size_t u = 0; u < U; u++) {                 /* validate first, touch nothing on error */
        int n = n_tok[u], t0 = c->q_len[u];
        if (n < 0 || n % 16 || t0 < 0 || t0 % 16 || t0 + n > s->Tcap || n > L) return -1;
        if (idx) {
            if (n > idx_stride) return -1;
            for (int i = 0; i < n; i++) {
                int r = idx[u * (size_t)idx_stride + i];
                if (r < 0 || r >= L) return -1;
                if (i && r <= idx[u * (size_t)idx_stride + i - 1]) return -1;
            }
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (size_t u = 0; u < U; u++) {
        int n = n_tok[u], t0 = c->q_len[u];
        uint32_t *Kc = c->Kc + u * pt_kc_words(s);
        uint32_t *Vc = c->Vc + u * pt_vc_words(s);
        uint16_t *Ks = c->Ks + u * (size_t)s->Tcap * NG, *Kz = c->Kz + u * (size_t)s->Tcap * NG;
        uint16_t *Vs = c->Vs + u * (size_t)s->Tcap * NG, *Vz = c->Vz + u * (size_t)s->Tcap * NG;
        int codes[128];
        for (int i = 0; i < n; i++) {
            int t = t0 + i, bit;
            size_t r = idx ? (size_t)idx[u * (size_t)idx_stride + i] : (size_t)i;
            /* the words of this token are rebuilt from zero (appends are whole words: multiples of 16 tokens) */
            for (int ch = 0; ch < D; ch++) {
                Kc[pt_k_slot(s, t, ch, &bit)] = 0;
                if (t % (32 / s->bits) == 0) Vc[pt_v_slot(s, t, ch, &bit)] = 0;
            }
            pt_quantize_row(s, K + (u * (size_t)L + r) * D, Ks + (size_t)t * NG, Kz + (size_t)t * NG, codes);
            for (int ch = 0; ch < D; ch++) {
                size_t w = pt_k_slot(s, t, ch, &bit);
                Kc[w] |= (uint32_t)codes[ch] << bit;
            }
            pt_quantize_row(s, V + (u * (size_t)L + r) * D, Vs + (size_t)t * NG, Vz + (size_t)t * NG, codes);
            for (int ch = 0; ch < D; ch++) {
                size_t w = pt_v_slot(s, t, ch, &bit);
                Vc[w] |= (uint32_t)codes[ch] << bit;
            }
        }
        c->q_len[u] = t0 + n;
    }
    return 0;
}

int ref_pt_unpack_codes(const ref_pt_shape *s, const ref_pt_cache *c, int unit, uint8_t *Kcodes, uint8_t *Vcodes)
{
    if (ref_pt_check_shape(s) || !c || unit < 0 || unit >= s->B * s->Hkv) return -1;
    const uint32_t *Kc = c->Kc + (size_t)unit * pt_kc_words(s);
    const uint32_t *Vc = c->Vc + (size_t)unit * pt_vc_words(s);
    const uint32_t mask = (1u << s->bits) - 1u;
    int T = c->q_len[unit];
    for (int t = 0; t < T; t++)
        for (int ch = 0; ch < s->D; ch++) {
            int bit;
            size_t w = pt_k_slot(s, t, ch, &bit);
            if (Kcodes) Kcodes[(size_t)t * s->D + ch] = (uint8_t)((Kc[w] >> bit) & mask);
            w = pt_v_slot(s, t, ch, &bit);
            if (Vcodes) Vcodes[(size_t)t * s->D + ch] = (uint8_t)((Vc[w] >> bit) & mask);
        }
    return 0;
}

int minikv_decode_attn_pt_ref(const ref_pt_shape *s, const uint16_t *q, const ref_pt_cache *c, float sm_scale,
                              uint16_t *out_f16, double *out_f64)
{
    if (ref_pt_check_shape(s) || !q || !c) return -1;
    const int D = s->D, G = s->G, NG = D / G, Hq = s->Hq, Hkv = s->Hkv, rep = Hq / Hkv;
    const uint32_t mask = (1u << s->bits) - 1u;
    const long NQ = (long)s->B * Hq;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bq = 0; bq < NQ; bq++) {
        size_t u = (size_t)(bq / Hq) * Hkv + (size_t)((bq % Hq) / rep);
        int T = c->q_len[u];
        if (T < 0) T = 0;
        if (T > s->Tcap) T = s->Tcap;
        const uint32_t *Kc = c->Kc + u * pt_kc_words(s);
        const uint32_t *Vc = c->Vc + u * pt_vc_words(s);
        const uint16_t *Ks = c->Ks + u * (size_t)s->Tcap * NG, *Kz = c->Kz + u * (size_t)s->Tcap * NG;
        const uint16_t *Vs = c->Vs + u * (size_t)s->Tcap * NG, *Vz = c->Vz + u * (size_t)s->Tcap * NG;
        double qd[128], o[128];
        for (int ch = 0; ch < D; ch++) { qd[ch] = (double)ref_f16_to_f32(q[(size_t)bq * D + ch]); o[ch] = 0.0; }
        double *a = (double *)malloc(sizeof(double) * (size_t)(T ? T : 1));
        if (!a) { fail = 1; continue; }
        for (int t = 0; t < T; t++) {                /* scores of the dequantized keys */
            double acc = 0.0;
            for (int ch = 0; ch < D; ch++) {
                int bit;
                size_t w = pt_k_slot(s, t, ch, &bit);
                double code = (double)((Kc[w] >> bit) & mask);
                size_t g = (size_t)t * NG + ch / G;
                acc += qd[ch] * (code * (double)ref_f16_to_f32(Ks[g]) + (double)ref_f16_to_f32(Kz[g]));
            }
            a[t] = (double)sm_scale * acc;
        }
        double mx = -INFINITY, sum = 0.0;            /* softmax */
        for (int t = 0; t < T; t++) if (a[t] > mx) mx = a[t];
        for (int t = 0; t < T; t++) { a[t] = exp(a[t] - mx); sum += a[t]; }
        for (int t = 0; t < T; t++) a[t] /= sum;
        for (int t = 0; t < T; t++)                  /* weighted dequantized values */
            for (int ch = 0; ch < D; ch++) {
                int bit;
                size_t w = pt_v_slot(s, t, ch, &bit);
                double code = (double)((Vc[w] >> bit) & mask);
                size_t g = (size_t)t * NG + ch / G;
                o[ch] += a[t] * (code * (double)ref_f16_to_f32(Vs[g]) + (double)ref_f16_to_f32(Vz[g]));
            }
        for (int ch = 0; ch < D; ch++) {
            if (out_f64) out_f64[(size_t)bq * D + ch] = o[ch];
            if (out_f16) out_f16[(size_t)bq * D + ch] = ref_f64_to_f16(o[ch]);
        }
        free(a);
    }
    return fail ? -1 : 0;
}
