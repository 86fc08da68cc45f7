/*
 * libminikv -- MiniKV decode-step attention over a 2-bit, adaptively evicted KV cache, for AMD MI355X
 * (gfx950).  C ABI: plain pointers and sizes, no C++ or framework types.
 *
 * What the calls compute is taken from the MiniKV paper: the 2-bit asymmetric group quantizer with
 * fp16 scale and zero-point and 16 codes per 32-bit word (Section 3.1.1, Section 3.3), the fp16
 * residual buffer that is compressed every n_r steps (Section 3.3, Algorithm 1 lines 9-15) and the
 * decode attention with dequantization fused into both products (Algorithm 1 lines 17-19), whose
 * result is softmax(q K^T * sm_scale) V of Appendix A eq. (1) over the compressed cache.  Two prefill-side
 * calls produce what those consume: the causal prompt attention that also returns every token's cumulative
 * attention score in linear memory (Section 3.2, Algorithm 1 line 2) and the heavy-hitter + recent-window
 * selection of the kept positions (Section 3.1.2, Algorithm 1 line 3), with the pyramid layer budget
 * (Section 3.1.3) as host arithmetic.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned; the library never
 *     allocates, frees or synchronises.  All work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream).  Lengths live in device memory so a decode loop never waits
 *     for the host.
 *   - fp16 = IEEE binary16 bit patterns (minikv_f16).  Inputs must be finite (no infinity, no NaN); every
 *     finite value is accepted.  minikv_decode_attn forms its matrix operands in fp16 and is fastest while
 *     |q_c * Ks| < 65504 for every channel and every V scale is below 4096 (a V group range below 12288);
 *     a (batch, KV head) unit that leaves this range is detected on the device and recomputed with
 *     range-normalised operands: same result to the stated tolerance, up to twice the time for that unit.
 *   - A "unit" is one (batch, KV head): u = b * Hkv + h.  Query head hq reads unit b*Hkv + hq/(Hq/Hkv).
 *   - Return value: MINIKV_OK (0) or a negative minikv_status; all checks happen on the host before
 *     anything is launched.  Values held in device memory (lengths, indices) are not validated; the
 *     kernels clamp lengths to the capacities.
 *
 * Shape rules: D == 128; G in {16, 32, 64, 128}; Tcap > 0 and Tcap % 128 == 0; Rcap % G == 0
 * (Rcap may be 0); Hq % Hkv == 0 and Hq / Hkv <= 8.
 *
 * Quantizer (Section 3.1.1 / 3.3).  For a group x_0..x_{G-1}: zero = min (fp16, -0 stored as +0),
 * scale = fp16_rne((max - min) / 3) with the subtraction and division in binary32,
 * code_i = clamp(rne((x_i - zero) * (1 / scale)), 0, 3) with each operation rounded to binary32 and
 * the reciprocal taken of the STORED fp16 scale (scale == 0: all codes 0), x_hat = code*scale + zero.
 * K groups are G consecutive retained tokens of one channel; V groups are G consecutive channels of one
 * token.
 *
 * Storage order (per unit; a storage choice made for coalesced 128-bit loads, the grouping above is
 * the paper's):
 *   Kc  uint32 [Tcap/128][4][64][4]   one word = 16 channels of ONE token: channel c of token t is in
 *       the token's word w = c/16 at bit 16*(c%2) + 2*((c%16)/2) (even channels in the low half-word,
 *       odd channels in the high one).  Word index = (t/128)*1024 + ((2*(t%2) + w/4)*64 + (t%128)/2)*4
 *       + w%4.
 *   Ks, Kz  fp16 [Tcap/G][D]          scale / zero of token group t/G.  Inside a row channel c sits at
 *       position ((q % NB)*(32/NB) + q/NB)*4 + c%4 with q = c/4 and NB = G/8: the 32 channel quads
 *       are dealt round-robin into NB bins, bin after bin.
 *   Vc  uint32 [Tcap/64][D][4]        one word = 16 consecutive tokens of ONE channel: token t is in
 *       block (t%64)/16 at bit 16*(t%2) + 2*((t%16)/2).  Word index = (t/64)*4*D + c*4 + (t%64)/16.
 *   Vs, Vz  fp16 [Tcap][D/G]          scale / zero of token t, channel group c/G.
 *   Rk, Rv  fp16 [Rcap][D]            residual rows, newest last.
 *   q_len, r_len  int32 [B*Hkv]       quantized tokens held (multiple of G) / residual rows held.
 */
#ifndef MINIKV_H
#define MINIKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MINIKV_ABI_VERSION 1

typedef uint16_t minikv_f16;

typedef enum {
    MINIKV_OK = 0,
    MINIKV_EINVAL = -1,        /* null or misaligned pointer, or a shape rule violated        */
    MINIKV_EUNSUPPORTED = -2,  /* D != 128, G not in the list, Hq/Hkv > 8                     */
    MINIKV_EWORKSPACE = -3,    /* workspace smaller than minikv_workspace_bytes()             */
    MINIKV_ELAUNCH = -4        /* the HIP runtime refused a launch (hipGetLastError != 0)     */
} minikv_status;

typedef struct minikv_shape {
    int32_t B, Hq, Hkv, D, G, Tcap, Rcap;
} minikv_shape;

typedef struct minikv_cache {
    uint32_t   *Kc;
    minikv_f16 *Ks, *Kz;
    uint32_t   *Vc;
    minikv_f16 *Vs, *Vz;
    int32_t    *q_len;
    minikv_f16 *Rk, *Rv;
    int32_t    *r_len;
} minikv_cache;

/* Index of a buffer for minikv_buffer_bytes(). */
typedef enum {
    MINIKV_BUF_KC = 0, MINIKV_BUF_KS, MINIKV_BUF_KZ, MINIKV_BUF_VC, MINIKV_BUF_VS, MINIKV_BUF_VZ,
    MINIKV_BUF_QLEN, MINIKV_BUF_RK, MINIKV_BUF_RV, MINIKV_BUF_RLEN
} minikv_buffer;

int         minikv_abi_version(void);
const char *minikv_strerror(int status);

/* Host-only helpers.  Bytes the caller must allocate for buffer `which` (a minikv_buffer) of a cache of
 * this shape, 0 on an invalid shape: per retained token 64 + 8*D/G bytes over the six packed buffers
 * (16 codes per 32-bit word plus an fp16 scale and zero-point per group, the storage arithmetic of the
 * paper's appendix on KV cache sizes), 4*D bytes per residual token, 4 bytes per length.
 * minikv_buffer_bytes is the same function under its earlier name.  minikv_workspace_bytes: bytes of the
 * split-K workspace of minikv_decode_attn. */
size_t minikv_cache_bytes(const minikv_shape *shape, int which);
size_t minikv_buffer_bytes(const minikv_shape *shape, int which);
size_t minikv_workspace_bytes(const minikv_shape *shape);

/* Algorithm 1 lines 3-5 (gather the retained tokens, quantize, pack) -- Section 3.1.1 / 3.3.
 * For every unit u: take n_tok[u] rows of K and V -- rows idx[u*idx_stride + i] (ascending) when idx is
 * not NULL, else rows 0..n_tok[u]-1 -- quantize them and write them at token offset q_len[u];
 * then q_len[u] += n_tok[u].
 *   K, V     fp16 [B*Hkv][L][D], contiguous                 (device, read)
 *   idx      int32 [B*Hkv][idx_stride] or NULL              (device, read)
 *   n_tok    int32 [B*Hkv], each a multiple of G, <= L      (device, read)
 *   max_tok  host-side upper bound of every n_tok[u] (sizes the launch; multiple of G, <= Tcap)
 * A unit whose q_len[u] + n_tok[u] would exceed Tcap, whose n_tok is not a positive multiple of G, or whose
 * n_tok exceeds max_tok is left unchanged. */
int kv_quantize_pack(const minikv_shape *shape, const minikv_f16 *K, const minikv_f16 *V, int64_t L,
                     const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, int32_t max_tok,
                     minikv_cache *cache, void *stream);

/* Algorithm 1 line 9: Rk[u][r_len[u]] = k_new[u], Rv likewise, r_len[u] += 1.
 *   k_new, v_new  fp16 [B*Hkv][D]                           (device, read)
 * A unit whose residual is already full (r_len == Rcap) is left unchanged: flush first. */
int kv_append_residual(const minikv_shape *shape, const minikv_f16 *k_new, const minikv_f16 *v_new,
                       minikv_cache *cache, void *stream);

/* Algorithm 1 lines 10-15: every unit with r_len[u] == Rcap (and room for Rcap more tokens) quantizes
 * its residual rows, appends them at q_len[u], then q_len[u] += Rcap and r_len[u] = 0.  Other units
 * are untouched.  The decision is taken on the device; calling it every step is cheap. */
int kv_flush_residual(const minikv_shape *shape, minikv_cache *cache, void *stream);

/* Algorithm 1 lines 17-19 / eq. (1):
 *   out[b][hq] = softmax(sm_scale * q[b][hq] . [K_hat ; Rk]^T) . [V_hat ; Rv]
 * over the q_len[u] quantized and r_len[u] residual tokens of unit u = b*Hkv + hq/(Hq/Hkv), one softmax
 * over the concatenation, fp32 accumulation, fp16 result.  A unit with no tokens gives zeros.
 *   q    fp16 [B][Hq][D]  (device, read)      out  fp16 [B][Hq][D]  (device, written)
 *   workspace  device scratch of at least minikv_workspace_bytes(shape) bytes, 16-byte aligned.  It must
 *              be ZERO-FILLED ONCE after allocation (it starts with per-unit ticket counters that every
 *              call returns to zero); beyond that its contents are private to the library.  Two calls
 *              that share a workspace must be ordered (same stream). */
int minikv_decode_attn(const minikv_shape *shape, const minikv_f16 *q, const minikv_cache *cache,
                       float sm_scale, minikv_f16 *out, void *workspace, size_t workspace_bytes,
                       void *stream);

/* The decode step in ONE launch, for callers that run kv_append_residual and minikv_decode_attn back to back (a
 * launch costs microseconds on this hardware however little it does): Algorithm 1 lines 9 and 17-19 together.
 * Equivalent to kv_append_residual(shape, k_new, v_new, cache) followed by minikv_decode_attn(...), same output
 * bit for bit, except for where the new residual lengths go:
 *   k_new, v_new  fp16 [B*Hkv][128], 16-byte aligned                       (device, read)
 *   r_len_next    int32 [B*Hkv], NOT cache->r_len                          (device, written)
 * Every wave of the launch reads cache->r_len when it starts, so the lengths after the append cannot go to the
 * same array: r_len_next[u] receives r_len[u] + 1 (r_len[u] unchanged when the buffer is full or the value is
 * out of range, as kv_append_residual leaves it), the new rows are written to their place in cache->Rk, Rv, and
 * the caller then uses r_len_next as the cache's r_len (swap the two pointers from step to step; no
 * synchronisation is involved).  kv_flush_residual and every other call take whichever array is current.
 * Where the flush goes: Algorithm 1 quantizes a residual that has just become full BETWEEN the append and the
 * attention (lines 10-15), which this entry point leaves no room for.  A loop built on it either runs the three
 * separate calls on the step that fills the residual, or calls kv_flush_residual at the start of the next step
 * (before that step's append): the cache ends up the same, and the one step that filled the residual has
 * attended to those tokens still in fp16 instead of quantized.
 * Other arguments, checks and status codes as minikv_decode_attn; MINIKV_EINVAL when r_len_next is null,
 * misaligned or equal to cache->r_len. */
int minikv_decode_step(const minikv_shape *shape, const minikv_f16 *q, const minikv_f16 *k_new, const minikv_f16 *v_new,
                       const minikv_cache *cache, int32_t *r_len_next, float sm_scale, minikv_f16 *out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): minikv_decode_attn with the split-K workspace held in a
 * device array of the library itself.  Same arguments, same kernel and same result as minikv_decode_attn
 * without `workspace` / `workspace_bytes`; the call allocates nothing.
 *   - The array (about 17.3 MB) exists once per GPU from the moment the library is loaded until the process
 *     ends.  It serves shapes with B * Hkv * ceil(Hq / Hkv / 4) <= minikv_static_workspace_units() (2048);
 *     larger shapes return MINIKV_EWORKSPACE and launch nothing.
 *   - Every call on one GPU uses that GPU's array: calls that may overlap on one GPU (different streams without
 *     an ordering between them) race; order them, or use minikv_decode_attn with a workspace per stream.
 *   - The first call on a GPU looks up the array's address and enqueues a small kernel on `stream` that
 *     zero-fills its ticket counters (a kernel, not a memset, so it may be captured); later calls enqueue the
 *     decode kernel only.  The device that is current at the call must be the one `stream` belongs to. */
size_t minikv_static_workspace_units(void);
int minikv_decode_attn_static(const minikv_shape *shape, const minikv_f16 *q, const minikv_cache *cache,
                              float sm_scale, minikv_f16 *out, void *stream);

/* ---------------------------------------------------------------------------------------------------------
 * Variant: PER-TOKEN quantized cache.  The paper's appendix on token-wise quantization quantizes keys and
 * values per token with 8, 4 and 2 bits (2 bits is the case it reports as failing, the reason MiniKV groups
 * keys per channel, Section 3.1.1), and its 4-bit per-token baseline is the one whose size the appendix on KV
 * cache compression ratios works out (16-bit values against 4-bit codes plus a 16-bit scale and zero-point per
 * head: a factor 3.76 at head dimension 128, i.e. bits = 4, G = 128 here).  These two calls build and read such
 * a cache, for comparisons against the 2-bit per-channel path above; there is no residual buffer (a token can
 * be quantized the moment it exists).
 *
 * Quantizer: as above with 2^bits - 1 steps, the G channels of ONE token forming a group, for K and V alike.
 * Shape rules: D == 128; G in {32, 64, 128}; bits in {2, 4, 8}; Tcap > 0, Tcap % 64 == 0; Hq % Hkv == 0,
 * Hq / Hkv <= 8.  Storage (per unit; cpw = 32 / bits codes per word, code i of a word at bits
 * [bits*i, bits*i + bits)):
 *   Kc uint32 [Tcap][D/cpw]  token major: word w of token t holds channels cpw*w ..
 *   Vc uint32 [Tcap/cpw][D]  channel major: word (t/cpw, c) holds cpw consecutive tokens of channel c
 *   Ks, Kz, Vs, Vz fp16 [Tcap][D/G];  q_len int32 [B*Hkv], a multiple of 16.
 * minikv_pt_cache_bytes takes the minikv_buffer index of a buffer (the residual entries give 0). */
typedef struct minikv_pt_shape {
    int32_t B, Hq, Hkv, D, G, bits, Tcap;
} minikv_pt_shape;

typedef struct minikv_pt_cache {
    uint32_t   *Kc;
    minikv_f16 *Ks, *Kz;
    uint32_t   *Vc;
    minikv_f16 *Vs, *Vz;
    int32_t    *q_len;
} minikv_pt_cache;

size_t minikv_pt_cache_bytes(const minikv_pt_shape *shape, int which);
size_t minikv_pt_workspace_bytes(const minikv_pt_shape *shape);

/* As kv_quantize_pack, per token: n_tok[u] rows (a multiple of 16, <= max_tok) are quantized and appended at
 * q_len[u] (a multiple of 16); a unit that breaks a rule is left unchanged. */
int kv_quantize_pack_pt(const minikv_pt_shape *shape, const minikv_f16 *K, const minikv_f16 *V, int64_t L,
                        const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, int32_t max_tok,
                        minikv_pt_cache *cache, void *stream);

/* out[b][hq] = softmax(sm_scale * q[b][hq] . K_hat^T) . V_hat (Appendix A eq. (1) on the dequantized cache)
 * over the q_len[u] tokens of unit u, fp32 accumulation, fp16 result; a unit without tokens gives zeros.
 * workspace: at least minikv_pt_workspace_bytes(shape) bytes, 16-byte aligned, no initial state required. */
int minikv_decode_attn_pt(const minikv_pt_shape *shape, const minikv_f16 *q, const minikv_pt_cache *cache,
                          float sm_scale, minikv_f16 *out, void *workspace, size_t workspace_bytes, void *stream);

/* Section 3.2 (selective flash attention) / Algorithm 1 line 2: causal attention of the prompt with itself that
 * also returns the cumulative attention score of every prompt token, in memory linear in L.  For batch b and
 * query head hq (reading KV head hq / (Hq/Hkv)), with P[i][j] = softmax_j(sm_scale * Q[i].K[j]) over j <= i:
 *   X_O[i]     = sum_j P[i][j] V[j]                      (fp16)
 *   lse[i]     = log sum_{j<=i} exp(sm_scale * Q[i].K[j])  (fp32, natural logarithm)
 *   A_cumul[j] = sum_{i>=j} P[i][j]                      (fp32; the rows kv_select_hh_rw takes)
 * Two passes as in Section 3.2: row blocks in parallel for X_O and lse, then column blocks in parallel that
 * recompute the scores and normalise them with lse.  fp16 operands, fp32 accumulation.
 *   Q          fp16 [B][Hq][L][128]                       (device, read)
 *   K, V       fp16 [B][Hkv][L][128]                      (device, read)
 *   X_O        fp16 [B][Hq][L][128]; lse fp32 [B][Hq][L]  (device, written)
 *   A_cumul    fp32 [B][Hq][L] or NULL (then only the first pass runs)   (device, written)
 *   workspace  device scratch of at least selective_flash_attn_workspace_bytes(B, Hkv, L) bytes, 16-byte
 *              aligned (a transposed copy of V: linear in L); contents private, no initial state required.
 * 1 <= L <= 2^23 (a head's rows are addressed with 32-bit byte offsets), Hq % Hkv == 0, B*Hkv <= 65535, pointers 16-byte aligned, sm_scale finite and > 0. */
size_t selective_flash_attn_workspace_bytes(int32_t B, int32_t Hkv, int64_t L);
int selective_flash_attn(int32_t B, int32_t Hq, int32_t Hkv, int64_t L, const minikv_f16 *Q, const minikv_f16 *K,
                         const minikv_f16 *V, float sm_scale, minikv_f16 *X_O, float *lse, float *A_cumul,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Section 3.1.2 (heavy hitters vs. recent window) / Algorithm 1 line 3: which prompt tokens a unit keeps.
 * The score of prompt token i of unit u is the binary32 sum, query heads in ascending order, of the rep
 * rows A_cumul[(u*rep + h)*L + i] (the cumulative attention score of Algorithm 1 line 2; under grouped-query
 * attention the heads of a group share one kept set, so their scores are added).  Kept: the n_rw[u] last
 * prompt tokens (the recent window) and, of the L - n_rw[u] others, the n_hh[u] with the largest score (the
 * heavy hitters); of equal scores the earlier position is kept.  idx[u*idx_stride + 0..n_tok[u]) receives
 * the kept positions in ascending order and n_tok[u] = n_hh[u] + n_rw[u]: exactly what kv_quantize_pack
 * takes (which in addition wants n_tok[u] to be a multiple of G: choose the budgets accordingly).
 *   units      number of (batch, KV head) units; rep = query heads per KV head (>= 1)
 *   A_cumul    fp32 [units*rep][L], finite, no NaN                        (device, read)
 *   n_hh, n_rw int32 [units]                                              (device, read)
 *   idx        int32 [units][idx_stride]; n_tok int32 [units]             (device, written)
 *   workspace  device scratch of at least kv_select_workspace_bytes(units, rep, L) bytes, 16-byte aligned;
 *              contents private, no initial state required (summed-score keys when rep > 1, and per
 *              4096-token chunk a histogram, a list of threshold candidates and counts: prompts of more than
 *              32768 tokens are selected by several workgroups per unit, in launches over (unit, chunk), so
 *              that a few long prompts still fill the chip; shorter ones by one workgroup per unit in one
 *              or two launches -- the result is the same).
 * A unit whose budgets are out of range (negative, n_rw > L, n_hh > L - n_rw, n_hh + n_rw > idx_stride)
 * gets n_tok[u] = 0 and its idx row is left alone.  L <= 2^30. */
size_t kv_select_workspace_bytes(int32_t units, int32_t rep, int64_t L);
int kv_select_hh_rw(int32_t units, int32_t rep, int64_t L, const float *A_cumul, const int32_t *n_hh,
                    const int32_t *n_rw, int32_t *idx, int64_t idx_stride, int32_t *n_tok, void *workspace,
                    size_t workspace_bytes, void *stream);

/* Section 3.1.3 (pyramid-like allocation) and the appendix paragraph on its details.  HOST arithmetic, no
 * device work: heavy-hitter budget of each of n_layers layers for an average budget x (tokens) and pyramid
 * depth d (the paper uses 7): one end layer gets x/d, the other 2x - x/d, the layers between are linearly
 * interpolated, so the mean stays x.  bottom_heavy != 0 gives layer 0 the large end (lower layers hold
 * more, as the section's text and the cited source say); 0 gives layer 0 the small end (the appendix
 * formula as printed).  n_layers == 1 gives x.
 *   budget  double [n_layers]                                             (HOST, written)
 * Returns MINIKV_EINVAL for n_layers < 1, d < 1, x < 0 or NaN, or a null pointer. */
int kv_pyramid_budget(int32_t n_layers, double x, int32_t d, int32_t bottom_heavy, double *budget);

#ifdef __cplusplus
}
#endif
#endif
