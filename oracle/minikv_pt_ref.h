/*
 * CPU oracle, second part: the PER-TOKEN quantized KV cache the paper compares against.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see minikv_ref.h).
 *
 * What it models.  The paper's baselines and its appendix on token-wise quantization quantize BOTH keys
 * and values per token: the channels of one token and head share a zero-point and a scale (fp16), with
 * 8-, 4- or 2-bit codes.  With 4 bits and one group per head this is the Q-Hitter-style baseline whose
 * compression factor the appendix on KV cache sizes gives as (d_head * 16) / (d_head * 4 + 2 * 16) = 3.76
 * for d_head = 128; with 2 bits it is the variant the appendix on token-wise quantization reports as
 * failing, because key outliers sit in channels (Section 3.1.1), which is why MiniKV quantizes keys per
 * channel.  There is no residual buffer: a token can be quantized the moment it is produced.
 *
 * Quantizer: the same asymmetric min/max quantizer as in minikv_ref.c with 2^bits - 1 steps:
 *   zero = group minimum (fp16, -0 stored as +0), scale = fp16_rne((max - min) / (2^bits - 1)) in binary32,
 *   code = clamp(rne((x - zero) * (1 / scale)), 0, 2^bits - 1), every operation a separately rounded
 *   binary32 operation, the reciprocal taken of the STORED scale, scale == 0 -> all codes 0.
 * Groups: G consecutive channels of one token (G in {32, 64, 128}), for K and for V alike.
 *
 * Storage order (per unit u = b*Hkv + h; cpw = 32 / bits codes per 32-bit word, code i of a word at bits
 * [bits*i, bits*i + bits)):
 *   Kc  uint32 [Tcap][D/cpw]      token major: word w of token t holds channels cpw*w .. cpw*w + cpw - 1
 *   Vc  uint32 [Tcap/cpw][D]      channel major: word (t/cpw, c) holds tokens cpw*(t/cpw) .. of channel c
 *   Ks, Kz, Vs, Vz  fp16 [Tcap][D/G]
 *   q_len int32 [B*Hkv]           tokens held, a multiple of 16
 *
 * Pins (tests/test_oracle_pt.py): half-step round-trip bound, codes 0 and 2^bits - 1 present, lossless
 * lattice, hand-packed words, the appendix's 3.76 compression factor, the 2-bit per-token codes against the
 * V path of minikv_ref.c (same grouping), fp64 brute-force attention from a numpy re-quantization, 8-bit
 * close to unquantized attention, and the ordering of errors on keys with outlier channels.
 */
#ifndef MINIKV_PT_REF_H
#define MINIKV_PT_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B, Hq, Hkv, D, G, bits, Tcap;
} ref_pt_shape;

typedef struct {
    uint32_t *Kc;
    uint16_t *Ks, *Kz;
    uint32_t *Vc;
    uint16_t *Vs, *Vz;
    int32_t  *q_len;
} ref_pt_cache;

/* 0 when: D == 128, G in {32, 64, 128}, bits in {2, 4, 8}, Tcap > 0, Tcap % 64 == 0, Hq % Hkv == 0. */
int ref_pt_check_shape(const ref_pt_shape *s);

/* Bytes one token of one head takes for K (the same for V): D*bits/8 code bytes + (D/G) * (2 + 2). */
size_t ref_pt_token_bytes(int D, int G, int bits);

/* Quantize n_tok[u] tokens (rows idx[u][i] when idx != NULL, else rows 0..n_tok[u]-1) of K and V, fp16
 * [B*Hkv][L][D], per token, and append them at q_len[u]; q_len[u] += n_tok[u].  n_tok[u] and q_len[u] must be
 * multiples of 16.  Returns 0, or -1 on a rule violation (nothing is touched then). */
int kv_quantize_pack_pt_ref(const ref_pt_shape *s, const uint16_t *K, const uint16_t *V, int64_t L,
                            const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, ref_pt_cache *c);

/* out[b][hq] = softmax(sm_scale * q[b][hq] . K_hat^T) . V_hat over the q_len[u] tokens of unit
 * u = b*Hkv + hq/(Hq/Hkv) (Appendix A eq. (1) on the dequantized cache), fp64 sums, one rounding to fp16.
 * out_f16 / out_f64 [B*Hq][D], either may be NULL.  A unit without tokens gives zeros. */
int minikv_decode_attn_pt_ref(const ref_pt_shape *s, const uint16_t *q, const ref_pt_cache *c, float sm_scale,
                              uint16_t *out_f16, double *out_f64);

/* Layout-free view for tests: codes[t][ch] of one unit (K and V). */
int ref_pt_unpack_codes(const ref_pt_shape *s, const ref_pt_cache *c, int unit, uint8_t *Kcodes, uint8_t *Vcodes);

#ifdef __cplusplus
}
#endif
#endif
