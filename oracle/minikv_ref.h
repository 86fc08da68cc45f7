/*
 * CPU oracle for MiniKV's decode-step attention over a 2-bit, evicted KV cache.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-precision-for-decisions /
 * double-precision-for-sums C implementation written straight from the paper (Section 3.1.1 and
 * Section 3.3 for the quantizer and the packing, Algorithm 1 "Decoding" for the residual buffer and
 * the attention, Appendix A eq. (1) for the attention definition).  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may use it; the GPU library never links or calls it, and this
 * directory shares no source, header, table or helper with the GPU library.
 *
 * Every pointer is a HOST pointer.  fp16 values travel as raw IEEE binary16 bit patterns (uint16_t).
 *
 * Storage order of the packed codes (a storage choice; the paper only fixes "16 two-bit codes per
 * 32-bit word", Section 3.3):
 *   K: one word = 16 channels of ONE token.  Channel c of token t lives in word  w = c / 16  of that
 *      token, at bit  16*(c%2) + 2*((c%16)/2)  (even channels fill the low half-word, odd channels
 *      the high half-word).  The 8 words of a token are laid out in tiles of 128 tokens:
 *      word index = tile*1024 + ((2*(t%2) + w/4)*64 + (t%128)/2)*4 + w%4,  tile = t/128.
 *   V: one word = 16 consecutive tokens of ONE channel.  Token t, channel c: block = (t%64)/16,
 *      bit 16*(t%2) + 2*((t%16)/2); tiles of 64 tokens:  word index = (t/64)*4*D + c*4 + block.
 *   Scale / zero-point: fp16, K [Tcap/G][D] per unit (token-group major), V [Tcap][D/G] per unit.
 *      Inside a K row channel c sits at ((q % NB)*(32/NB) + q/NB)*4 + c%4 with q = c/4, NB = G/8
 *      (the 32 channel quads dealt round-robin into NB bins).
 *
 * Pins (tests/ with -m "not gpu"): round-trip half-step bound, code 0/3 presence, lossless lattice,
 * fp64 arg-min brute force with explicit ties, hand-derived packed words, Appendix I size arithmetic,
 * fp64 exact attention on a separately dequantized cache, softmax rows summing to 1, T=0 and r=0
 * special cases, uniform-weight case, GQA == replicated MHA, unit permutation; for the token selection:
 * a library sort with explicit tie keys, monotone / constant score closed forms, exhaustive tiny cases,
 * boundary budgets, pre-summed heads; for the pyramid budget: mean, end points, linearity; for the prefill
 * attention: a numpy matmul + softmax, equal keys (harmonic-number column sums), rows summing to one,
 * first and last token, GQA == replicated MHA.  No function here is "parity unpinned".
 */
#ifndef MINIKV_REF_H
#define MINIKV_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B, Hq, Hkv, D, G, Tcap, Rcap;
} ref_shape;

typedef struct {
    uint32_t *Kc;   /* [B*Hkv][Tcap/128][1024] words                       */
    uint16_t *Ks;   /* [B*Hkv][Tcap/G][D] fp16                             */
    uint16_t *Kz;   /* [B*Hkv][Tcap/G][D] fp16                             */
    uint32_t *Vc;   /* [B*Hkv][Tcap/64][D][4] words                        */
    uint16_t *Vs;   /* [B*Hkv][Tcap][D/G] fp16                             */
    uint16_t *Vz;   /* [B*Hkv][Tcap][D/G] fp16                             */
    int32_t  *q_len;/* [B*Hkv] quantized tokens held, multiple of G        */
    uint16_t *Rk;   /* [B*Hkv][Rcap][D] fp16 residual keys                 */
    uint16_t *Rv;   /* [B*Hkv][Rcap][D] fp16 residual values               */
    int32_t  *r_len;/* [B*Hkv] residual tokens held, 0..Rcap               */
} ref_cache;

/* IEEE binary16 <-> binary32/64, round-to-nearest-even, subnormals kept. */
float    ref_f16_to_f32(uint16_t h);
uint16_t ref_f32_to_f16(float f);
uint16_t ref_f64_to_f16(double x);

/* 0 when the shape obeys: D==128, G in {16,32,64,128}, Tcap%128==0, Tcap>0, Rcap%G==0, Hq%Hkv==0. */
int ref_check_shape(const ref_shape *s);

/* Section 3.1.1 / 3.3 + Algorithm 1 line 4: quantize n_tok[u] tokens of K and V (rows idx[u][i] of the
 * source when idx != NULL, else rows 0..n_tok[u]-1) and append them at token offset q_len[u];
 * q_len[u] += n_tok[u].  K, V: fp16 [B*Hkv][L][D].  Returns 0, or -1 on a rule violation. */
int kv_quantize_pack_ref(const ref_shape *s, const uint16_t *K, const uint16_t *V, int64_t L,
                         const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, ref_cache *c);

/* Algorithm 1 line 9: append one token per unit to the residual; a full unit is left unchanged. */
int kv_append_residual_ref(const ref_shape *s, const uint16_t *k_new, const uint16_t *v_new,
                           ref_cache *c);

/* Algorithm 1 lines 10-15: every unit whose residual holds exactly Rcap tokens quantizes it,
 * appends it to the packed cache and empties the residual. */
int kv_flush_residual_ref(const ref_shape *s, ref_cache *c);

/* Algorithm 1 lines 17-19 with eq. (1)'s scale passed in as sm_scale.
 * out_f16 [B*Hq][D] (may be NULL), out_f64 [B*Hq][D] un-rounded (may be NULL),
 * probs [B*Hq][Tcap+Rcap] softmax weights, quantized tokens first then residual (may be NULL). */
int minikv_decode_attn_ref(const ref_shape *s, const uint16_t *q, const ref_cache *c, float sm_scale,
                           uint16_t *out_f16, double *out_f64, double *probs);

/* Section 3.2 (the two outputs of the selective attention kernel) + Algorithm 1 line 2, with the attention
 * of Appendix A eq. (1) restricted to the causal part (query i sees keys 0..i): for every batch b and query
 * head hq (reading KV head hq / (Hq/Hkv)), in fp64 from the fp16 inputs,
 *   P[i][j]    = softmax_j(sm_scale * Q[i].K[j]),  j <= i
 *   X_O[i]     = sum_j P[i][j] V[j]                         (XO_f16: rounded once to fp16; XO_f64: not rounded)
 *   lse[i]     = log sum_j exp(sm_scale * Q[i].K[j])        (natural logarithm)
 *   A_cumul[j] = sum_{i >= j} P[i][j]                       (column sums of the attention matrix)
 * Q [B][Hq][L][D], K, V [B][Hkv][L][D] fp16; outputs [B][Hq][L][D] and [B][Hq][L]; any output may be NULL.
 * The full matrix is never stored (one row at a time), but nothing is tiled or reordered.
 * Returns 0, or -1 on bad arguments. */
int selective_flash_attn_ref(int32_t B, int32_t Hq, int32_t Hkv, int64_t L, int32_t D, const uint16_t *Q,
                             const uint16_t *K, const uint16_t *V, float sm_scale, uint16_t *XO_f16,
                             double *XO_f64, double *lse, double *A_cumul);

/* The same quantities for a list of query rows of ONE head (Q, K, V [L][D] of that head), for checks at sizes
 * where the whole matrix is out of reach: xo [n_rows][D] (fp64), lse [n_rows], and p_tail [n_rows][tail] = the
 * row's weights of the last `tail` keys (zero for keys after the row).  Any output may be NULL. */
int selective_flash_attn_rows_ref(int64_t L, int32_t D, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                                  float sm_scale, const int64_t *rows, int32_t n_rows, double *xo, double *lse,
                                  double *p_tail, int32_t tail);

/* Section 3.1.2 (heavy hitters and recent window) + Algorithm 1 line 3.  For every unit u the score of
 * prompt token i is the binary32 sum, query heads in ascending order, of the rep rows
 * A_cumul[(u*rep + h)*L + i].  Kept tokens: the n_rw[u] last prompt tokens (recent window) and, of the
 * L - n_rw[u] others, the n_hh[u] with the largest score; of equal scores the earlier position wins.
 * idx[u*idx_stride + 0..n_tok[u]) receives the kept positions in ascending order, n_tok[u] = n_hh[u] +
 * n_rw[u].  A unit whose budgets are out of range (negative, n_rw > L, n_hh > L - n_rw, or
 * n_hh + n_rw > idx_stride) gets n_tok[u] = 0 and its idx row is left alone.  Scores must not be NaN.
 * Returns 0, or -1 on bad arguments. */
int kv_select_hh_rw_ref(int32_t units, int32_t rep, int64_t L, const float *A_cumul,
                        const int32_t *n_hh, const int32_t *n_rw, int32_t *idx, int64_t idx_stride,
                        int32_t *n_tok);

/* Section 3.1.3, pyramid-like allocation, and its appendix paragraph: heavy-hitter budget of each of
 * n_layers layers for an average budget x and pyramid depth d: one end layer gets x/d, the other
 * 2x - x/d, the layers between are linearly interpolated.  bottom_heavy != 0 gives layer 0 the large end
 * (what the prose and the cited source say), 0 the small end (the appendix formula as printed).
 * n_layers == 1 gives x.  Returns 0, or -1 on bad arguments (n_layers < 1, d < 1, x < 0). */
int kv_pyramid_budget_ref(int32_t n_layers, double x, int32_t d, int32_t bottom_heavy, double *budget);

/* Layout-free views for tests: codes[unit][t][ch] (0..3) and the dequantized values code*s+z. */
int ref_unpack_codes(const ref_shape *s, const ref_cache *c, int unit, uint8_t *Kcodes, uint8_t *Vcodes);
int ref_dequant(const ref_shape *s, const ref_cache *c, int unit, double *Khat, double *Vhat);

/* Position of channel c inside a K scale / zero row (see the storage order above). */
int ref_k_meta_pos(int G, int c);

/* Appendix I: bytes of one packed group of G codes with its fp16 scale and zero-point. */
size_t ref_group_bytes(int G);

#ifdef __cplusplus
}
#endif
#endif
