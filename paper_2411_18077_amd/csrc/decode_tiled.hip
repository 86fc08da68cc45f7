// Wave-tiled decode attention over the packed 2-bit cache (gfx950, wave64).
//
// Computes Algorithm 1 lines 17-19 of the MiniKV paper (scores of the dequantized keys and the fp16
// residual keys, one softmax, weighted dequantized + residual values; eq. (1) scale passed in) with the
// dequantization folded into both products (Section 3.3, "fused unpacking and multiplication"):
//
//   score_t = sum_c (q_c * Ks[g,c]) * code_tc  +  sum_c q_c * Kz[g,c]          g = t / G
//   out_c   = sum_t (p_t * Vs[t,gc]) * code_tc +  sum_t p_t * Vz[t,gc]         gc = c / G
//
// so the inner products run over the raw 2-bit codes and the scales move onto the small operands.
//
// Work split: one workgroup (4 waves) per (unit, token chunk); inside it every wave is independent and
// walks "passes" of 128 tokens with its own online-softmax state; waves merge through LDS at the end and
// the workgroup writes one split-K partial (merged by merge_kernel).
//
// One pass, lane l of the wave:
//   K phase: the lane owns tokens 2l and 2l+1.  Four 128-bit loads bring their 2 x 8 code words.  The
//     wave builds, per K group of the pass, a table qs[g][c] = q_c * Ks[g,c] in LDS as an fp16 pair
//     (hi, lo) whose sum is the exact product, pre-multiplied by 4^-j (see below).  Codes are NOT
//     converted: (word & (0x00030003 << 2j)) is used directly as two fp16 SUBNORMALS code * 4^j * 2^-24
//     (j <= 4 keeps the field inside the mantissa; fields 5..7 come from the word shifted right by 6).
//     The 4-head x 4-channel block products go either to v_mfma_f32_4x4x4f16 (16 blocks = 64 tokens per
//     instruction, lane = token, 4 result registers = 4 query heads) or to v_dot2_f32_f16.
//   softmax: per-head wave maximum, lazy rescale of the accumulators, p = exp2(score - m).
//   V phase: the lane owns channels l and l+64.  ps[gc][h][t] = p * Vs * 2^4 * 4^-j(t) goes to LDS as
//     fp16; the V words (16 tokens of one channel, even tokens in the low half-word) are masked the same
//     way and multiplied 4 tokens x 4 heads at a time.  The zero-point term is accumulated per lane in
//     fp32 and reduced once per chunk.
//
// Input domain implied by the fp16 operands: |q * Ks| < 65504 and Vs < 4096 (V group range < 12288).
#include "decode_common.h"

#include <hip/hip_fp16.h>

namespace minikv {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr int kNH = 4;                 // query-head slots per workgroup (rows of the 4x4x4 blocks)
constexpr int kPass = 128;             // tokens per wave pass
constexpr int kQsG = 32 * 16 + 16;     // halfs per K-group table: 32 k-steps x (4 heads x 4 ch) + pad
constexpr int kPsH = kPass + 4;        // halfs per (channel group, head) row of ps, padded
constexpr int kPsG = kNH * kPsH;       // halfs per channel group of ps (528: shifts 8 banks)

__device__ inline h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ inline uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }
__device__ inline float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// field j (0..7) of a half-word pair -> (shift inside the mantissa, use the >>6 copy?)
__host__ __device__ constexpr int fld_shift(int j) { return j <= 4 ? 2 * j : 2 * (j - 3); }
__host__ __device__ constexpr bool fld_shifted(int j) { return j > 4; }
// 4^-(shift/2): what the small operand is pre-multiplied by so that the masked subnormal needs no shift
__device__ inline float fld_scale(int j) { return 1.0f / (float)(1 << fld_shift(j)); }

__device__ inline h2 field(uint32_t w, uint32_t w6, int j)
{
    return as_h2((fld_shifted(j) ? w6 : w) & (0x00030003u << fld_shift(j)));
}

__device__ inline float wave_max64(float v)
{
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float wave_sum64(float v)
{
    for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int N> struct Words { uint32_t v[N]; };
template <int N> __device__ inline Words<N> load_words(const void *p)
{
    Words<N> r;
    if constexpr (N == 1) { r.v[0] = *reinterpret_cast<const uint32_t *>(p); }
    else if constexpr (N == 2) { uint2 t = *reinterpret_cast<const uint2 *>(p); r.v[0] = t.x; r.v[1] = t.y; }
    else {
        for (int i = 0; i < N / 4; i++) {
            uint4 t = reinterpret_cast<const uint4 *>(p)[i];
            r.v[4 * i] = t.x; r.v[4 * i + 1] = t.y; r.v[4 * i + 2] = t.z; r.v[4 * i + 3] = t.w;
        }
    }
    return r;
}

// ------------------------------------------------------------------------------------------------
// fp16 residual chunk: Algorithm 1's R_K t_Q^T and A_unquant R_V, plain vector-ALU code.
// Wave w takes tokens [64*(w + 4i), +64); lane = token for the scores, lane = channel pair for the values.
__device__ void residual_chunk(const DecArgs &a, int u, int bq0, int nheads, int R, _Float16 *lds)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    _Float16 *qh = lds;                                   // [kNH][128] halfs, shared by the workgroup
    float *pw = reinterpret_cast<float *>(lds + kNH * kD) + wave * (kNH * 64);   // [kNH][64] per wave
    for (int i = tid; i < kNH * kD; i += 256) {
        const int h = i / kD;
        qh[i] = (h < nheads) ? __builtin_bit_cast(_Float16, a.q[(size_t)(bq0 + h) * kD + i % kD]) : (_Float16)0.f;
    }
    __syncthreads();
    const uint16_t *Rk = a.Rk + (size_t)u * a.Rcap * kD;
    const uint16_t *Rv = a.Rv + (size_t)u * a.Rcap * kD;

    float m[kNH], l[kNH], o0[kNH], o1[kNH];
    for (int h = 0; h < kNH; h++) { m[h] = -1e30f; l[h] = 0.f; o0[h] = 0.f; o1[h] = 0.f; }

    for (int t0 = wave * 64; t0 < R; t0 += 256) {
        const int t = t0 + lane;
        const bool valid = t < R;
        float acc[kNH] = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            const uint4 *row = reinterpret_cast<const uint4 *>(Rk + (size_t)t * kD);
#pragma unroll 4
            for (int i = 0; i < 16; i++) {
                const uint4 kk = row[i];
                const uint32_t kw[4] = {kk.x, kk.y, kk.z, kk.w};
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    const u4 qq = *reinterpret_cast<const u4 *>(qh + h * kD + i * 8);
#pragma unroll
                    for (int p = 0; p < 4; p++)
                        acc[h] = __builtin_amdgcn_fdot2(as_h2(qq[p]), as_h2(kw[p]), acc[h], false);
                }
            }
        }
        float p[kNH];
        bool grow = false;
        float mn[kNH];
        for (int h = 0; h < kNH; h++) {
            const float s = valid ? acc[h] * a.c1 : -INFINITY;
            mn[h] = fmaxf(m[h], wave_max64(s));
            grow |= mn[h] > m[h];
            acc[h] = s;
        }
        if (grow)
            for (int h = 0; h < kNH; h++) {
                const float sc = exp2f(m[h] - mn[h]);
                l[h] *= sc; o0[h] *= sc; o1[h] *= sc;
                m[h] = mn[h];
            }
        for (int h = 0; h < kNH; h++) {
            p[h] = exp2f(acc[h] - m[h]);
            l[h] += p[h];
            pw[h * 64 + lane] = p[h];
        }
        __builtin_amdgcn_wave_barrier();
        const int nt = min(64, R - t0);
        for (int tt = 0; tt < nt; tt++) {
            const h2 v = as_h2(*reinterpret_cast<const uint32_t *>(Rv + (size_t)(t0 + tt) * kD + 2 * lane));
            const float v0 = (float)v[0], v1 = (float)v[1];
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                const float ph = pw[h * 64 + tt];
                o0[h] += ph * v0;
                o1[h] += ph * v1;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // merge the four waves
    __syncthreads();
    float *mo = reinterpret_cast<float *>(lds);            // [4 waves][kNH][128]
    float *mm = mo + 4 * kNH * kD;                         // [4][kNH]
    float *ml = mm + 4 * kNH;
    for (int h = 0; h < kNH; h++) {
        mo[(wave * kNH + h) * kD + 2 * lane] = o0[h];
        mo[(wave * kNH + h) * kD + 2 * lane + 1] = o1[h];
        const float ls = wave_sum64(l[h]);
        if (lane == 0) { mm[wave * kNH + h] = m[h]; ml[wave * kNH + h] = ls; }
    }
    __syncthreads();
    const int c = tid & 127;
    for (int h = tid >> 7; h < nheads; h += 2) {
        float M = -1e30f;
        for (int w = 0; w < 4; w++) M = fmaxf(M, mm[w * kNH + h]);
        float L = 0.f, O = 0.f;
        for (int w = 0; w < 4; w++) {
            const float sc = exp2f(mm[w * kNH + h] - M);
            L += ml[w * kNH + h] * sc;
            O += mo[(w * kNH + h) * kD + c] * sc;
        }
        float *pp = partial_ptr(a, bq0 + h, a.nchunk);
        pp[4 + c] = O;
        if (c == 0) { pp[0] = M; pp[1] = L; }
    }
}

// ------------------------------------------------------------------------------------------------
template <int G, bool MFMA, bool LO>
__global__ __launch_bounds__(256) void decode_tiled_kernel(DecArgs a)
{
    constexpr int NG = kPass / G > 0 ? kPass / G : 1;      // K groups per pass (G=128: 1)
    constexpr int LPG = 64 / NG;                           // lanes per K group (= G/2)
    constexpr int CPL = kD / LPG;                          // channels per lane in the table build
    constexpr int NPR = CPL / 2;                           // channel pairs per lane
    constexpr int NCG = kD / G;                            // V channel groups
    constexpr int WAVE_HALFS = (LO ? 2 : 1) * NG * kQsG + NCG * kPsG;

    extern __shared__ __attribute__((aligned(16))) _Float16 lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = blockIdx.y, ch = blockIdx.x, hs = blockIdx.z;
    const int b = u / a.Hkv, kvh = u % a.Hkv;
    const int bq0 = b * a.Hq + kvh * a.rep + hs * kNH;
    const int nheads = min(kNH, a.rep - hs * kNH);

    if (ch == a.nchunk) {
        const int R = clampi(a.r_len[u], 0, a.Rcap);
        if (R == 0) return;
        residual_chunk(a, u, bq0, nheads, R, lds);
        return;
    }
    const int T = clampi(a.q_len[u], 0, a.Tcap);
    const int t_begin = ch * a.chunk;
    const int t_end = min(T, t_begin + a.chunk);
    if (t_begin >= t_end) return;

    _Float16 *qs_hi = lds + wave * WAVE_HALFS;
    _Float16 *qs_lo = qs_hi + NG * kQsG;                   // only used when LO
    _Float16 *ps = qs_hi + (LO ? 2 : 1) * NG * kQsG;

    const uint32_t *Kc = a.Kc + (size_t)u * kc_words(a.Tcap);
    const uint32_t *Vc = a.Vc + (size_t)u * vc_words(a.Tcap);
    const uint16_t *Ks = a.Ks + (size_t)u * (a.Tcap / G) * kD;
    const uint16_t *Kz = a.Kz + (size_t)u * (a.Tcap / G) * kD;
    const uint16_t *Vs = a.Vs + (size_t)u * a.Tcap * NCG;
    const uint16_t *Vz = a.Vz + (size_t)u * a.Tcap * NCG;

    // ---- per-lane constants of the table build: this lane's CPL channels of every head's query
    const int gl = lane / LPG;                             // K group (of the pass) this lane serves AND
                                                           // the group of its own two tokens
    const int c0 = (lane % LPG) * CPL;                     // first channel of the lane's slice
    h2 qraw[kNH][NPR], qscl[kNH][NPR];
#pragma unroll
    for (int h = 0; h < kNH; h++)
#pragma unroll
        for (int p = 0; p < NPR; p++) {
            uint32_t bits = 0;
            if (h < nheads) bits = *reinterpret_cast<const uint32_t *>(a.q + (size_t)(bq0 + h) * kD + c0 + 2 * p);
            qraw[h][p] = as_h2(bits);
            // channel pair (c, c+1), c even, sits in field j = (c % 16) / 2 of its K word
            const float sc = fld_scale(((c0 + 2 * p) & 15) >> 1);
            qscl[h][p] = qraw[h][p] * (_Float16)sc;
        }

    // V side: this lane's two channels and their channel groups
    const int cg0 = lane / G;                              // G=128: 0
    const int cg1 = (lane + 64) / G;

    float m[kNH], l_lane[kNH];
    f4 O0 = {0.f, 0.f, 0.f, 0.f}, O1 = {0.f, 0.f, 0.f, 0.f};   // channel lane / lane+64, 4 heads each
    float oz[kNH][NCG];
#pragma unroll
    for (int h = 0; h < kNH; h++) {
        m[h] = -1e30f; l_lane[h] = 0.f;
#pragma unroll
        for (int g = 0; g < NCG; g++) oz[h][g] = 0.f;
    }

    const float kscale = a.c1 * 16777216.0f;               // undo the 2^-24 of the subnormal code fields
    const int npass = (t_end - t_begin + kPass - 1) / kPass;

    for (int pass = wave; pass < npass; pass += 4) {
        const int tp = t_begin + pass * kPass;             // multiple of 128
        const bool valid = tp + 2 * lane < t_end;          // both tokens of the lane (t_end % 16 == 0)

        // ---------------- loads of the pass
        const u4 *ktile = reinterpret_cast<const u4 *>(Kc + (size_t)(tp >> 7) * 1024);
        u4 kw[4];
#pragma unroll
        for (int i = 0; i < 4; i++) kw[i] = ktile[i * 64 + lane];
        const u4 *vtile = reinterpret_cast<const u4 *>(Vc + (size_t)(tp >> 6) * (4 * kD));
        u4 vw[2][2];                                       // [channel half][64-token tile]
#pragma unroll
        for (int tl = 0; tl < 2; tl++) {
            vw[0][tl] = vtile[tl * kD + lane];
            vw[1][tl] = vtile[tl * kD + lane + 64];
        }
        const bool gvalid = tp + gl * G < t_end;
        Words<NPR> ksw, kzw;
        {
            const size_t go = ((size_t)(tp / G) + (gvalid ? gl : 0)) * kD + c0;
            ksw = load_words<NPR>(Ks + go);
            kzw = load_words<NPR>(Kz + go);
        }
        Words<NCG> vsw, vzw;                               // 2 tokens x NCG fp16 = NCG words
        {
            const size_t vo = (size_t)(valid ? tp + 2 * lane : tp) * NCG;
            vsw = load_words<NCG>(Vs + vo);
            vzw = load_words<NCG>(Vz + vo);
        }

        // ---------------- qs table of the pass's K groups, and qz = sum_c q_c Kz[g,c]
        float qz[kNH] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < NPR; p++) {
            const h2 ks2 = as_h2(ksw.v[p]), kz2 = as_h2(kzw.v[p]);
            const int c = c0 + 2 * p;                      // even channel of the pair
            const int off = gl * kQsG + (c >> 2) * 16 + (c & 3);
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                const h2 hi = qscl[h][p] * ks2;
                *reinterpret_cast<h2 *>(qs_hi + off + h * 4) = hi;
                if constexpr (LO) {
                    const h2 lo = __builtin_elementwise_fma(qscl[h][p], ks2, -hi);
                    *reinterpret_cast<h2 *>(qs_lo + off + h * 4) = lo;
                }
                qz[h] = __builtin_amdgcn_fdot2(qraw[h][p], kz2, qz[h], false);
            }
        }
#pragma unroll
        for (int h = 0; h < kNH; h++)
            for (int o = LPG / 2; o; o >>= 1) qz[h] += __shfl_xor(qz[h], o);
        __builtin_amdgcn_wave_barrier();

        // ---------------- K products: scores of tokens 2*lane, 2*lane+1 for the 4 heads
        f4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        {
            const _Float16 *th = qs_hi + gl * kQsG;
            const _Float16 *tl = qs_lo + gl * kQsG;
#pragma unroll
            for (int w = 0; w < 8; w++) {
                const uint32_t w0 = kw[w >> 2][w & 3], w1 = kw[2 + (w >> 2)][w & 3];
                const uint32_t w0s = w0 >> 6, w1s = w1 >> 6;
#pragma unroll
                for (int sq = 0; sq < 4; sq++) {
                    const int s = 4 * w + sq;
                    const h2 x00 = field(w0, w0s, 2 * sq), x01 = field(w0, w0s, 2 * sq + 1);
                    const h2 x10 = field(w1, w1s, 2 * sq), x11 = field(w1, w1s, 2 * sq + 1);
                    if constexpr (MFMA) {
                        const h4 b0 = {x00[0], x00[1], x01[0], x01[1]};
                        const h4 b1 = {x10[0], x10[1], x11[0], x11[1]};
                        const h4 ah = *reinterpret_cast<const h4 *>(th + s * 16 + (lane & 3) * 4);
                        acc0 = __builtin_amdgcn_mfma_f32_4x4x4f16(ah, b0, acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_4x4x4f16(ah, b1, acc1, 0, 0, 0);
                        if constexpr (LO) {
                            const h4 al = *reinterpret_cast<const h4 *>(tl + s * 16 + (lane & 3) * 4);
                            acc0 = __builtin_amdgcn_mfma_f32_4x4x4f16(al, b0, acc0, 0, 0, 0);
                            acc1 = __builtin_amdgcn_mfma_f32_4x4x4f16(al, b1, acc1, 0, 0, 0);
                        }
                    } else {
#pragma unroll
                        for (int h = 0; h < kNH; h++) {
                            const u4 ah = *reinterpret_cast<const u4 *>(th + s * 16 + h * 4 - 4 * (h & 1)) ;
                            // two heads share one 128-bit read: (h even: words 0,1 ; h odd: words 2,3)
                            const h2 a0 = as_h2(ah[2 * (h & 1)]), a1 = as_h2(ah[2 * (h & 1) + 1]);
                            acc0[h] = __builtin_amdgcn_fdot2(a0, x00, acc0[h], false);
                            acc0[h] = __builtin_amdgcn_fdot2(a1, x01, acc0[h], false);
                            acc1[h] = __builtin_amdgcn_fdot2(a0, x10, acc1[h], false);
                            acc1[h] = __builtin_amdgcn_fdot2(a1, x11, acc1[h], false);
                            if constexpr (LO) {
                                const u4 al = *reinterpret_cast<const u4 *>(tl + s * 16 + h * 4 - 4 * (h & 1));
                                const h2 l0 = as_h2(al[2 * (h & 1)]), l1 = as_h2(al[2 * (h & 1) + 1]);
                                acc0[h] = __builtin_amdgcn_fdot2(l0, x00, acc0[h], false);
                                acc0[h] = __builtin_amdgcn_fdot2(l1, x01, acc0[h], false);
                                acc1[h] = __builtin_amdgcn_fdot2(l0, x10, acc1[h], false);
                                acc1[h] = __builtin_amdgcn_fdot2(l1, x11, acc1[h], false);
                            }
                        }
                    }
                }
            }
        }

        // ---------------- online softmax (per head, wave-wide maximum)
        float s0[kNH], s1[kNH], mn[kNH];
        bool grow = false;
#pragma unroll
        for (int h = 0; h < kNH; h++) {
            const float zz = qz[h] * a.c1;
            s0[h] = valid ? acc0[h] * kscale + zz : -INFINITY;
            s1[h] = valid ? acc1[h] * kscale + zz : -INFINITY;
            mn[h] = fmaxf(m[h], wave_max64(fmaxf(s0[h], s1[h])));
            grow |= mn[h] > m[h];
        }
        if (grow) {
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                const float sc = exp2f(m[h] - mn[h]);
                l_lane[h] *= sc;
                O0[h] *= sc;
                O1[h] *= sc;
#pragma unroll
                for (int g = 0; g < NCG; g++) oz[h][g] *= sc;
                m[h] = mn[h];
            }
        }

        // ---------------- weights, ps table, zero-point term
        {
            // token 2*lane is field j = lane & 7 of its V word (low half), 2*lane+1 the high half
            const float vsc = 16.0f * fld_scale(lane & 7);
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                const float p0 = exp2f(s0[h] - m[h]), p1 = exp2f(s1[h] - m[h]);   // masked lanes: 0
                l_lane[h] += p0 + p1;
#pragma unroll
                for (int g = 0; g < NCG; g++) {
                    // words hold [token 2l: NCG halfs][token 2l+1: NCG halfs]
                    const int i0 = g, i1 = NCG + g;
                    const h2 sw0 = as_h2(vsw.v[i0 >> 1]), sw1 = as_h2(vsw.v[i1 >> 1]);
                    const h2 zw0 = as_h2(vzw.v[i0 >> 1]), zw1 = as_h2(vzw.v[i1 >> 1]);
                    const float vs0 = valid ? (float)sw0[i0 & 1] : 0.f, vs1 = valid ? (float)sw1[i1 & 1] : 0.f;
                    const float vz0 = valid ? (float)zw0[i0 & 1] : 0.f, vz1 = valid ? (float)zw1[i1 & 1] : 0.f;
                    const h2 pv = {(_Float16)(p0 * vs0 * vsc), (_Float16)(p1 * vs1 * vsc)};
                    *reinterpret_cast<h2 *>(ps + g * kPsG + h * kPsH + 2 * lane) = pv;
                    oz[h][g] += p0 * vz0 + p1 * vz1;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();

        // ---------------- V products: channels lane and lane+64, 4 heads, 4 tokens per step
        {
            const _Float16 *pa0 = ps + cg0 * kPsG + (MFMA ? (lane & 3) * kPsH : 0);
            const _Float16 *pa1 = ps + cg1 * kPsG + (MFMA ? (lane & 3) * kPsH : 0);
#pragma unroll
            for (int blk = 0; blk < 8; blk++) {
                const uint32_t v0 = vw[0][blk >> 2][blk & 3], v1 = vw[1][blk >> 2][blk & 3];
                const uint32_t v0s = v0 >> 6, v1s = v1 >> 6;
#pragma unroll
                for (int ks = 0; ks < 4; ks++) {
                    const int tok = 16 * blk + 4 * ks;
                    const h2 x00 = field(v0, v0s, 2 * ks), x01 = field(v0, v0s, 2 * ks + 1);
                    const h2 x10 = field(v1, v1s, 2 * ks), x11 = field(v1, v1s, 2 * ks + 1);
                    if constexpr (MFMA) {
                        const h4 b0 = {x00[0], x00[1], x01[0], x01[1]};
                        const h4 b1 = {x10[0], x10[1], x11[0], x11[1]};
                        const h4 a0 = *reinterpret_cast<const h4 *>(pa0 + tok);
                        const h4 a1 = *reinterpret_cast<const h4 *>(pa1 + tok);
                        O0 = __builtin_amdgcn_mfma_f32_4x4x4f16(a0, b0, O0, 0, 0, 0);
                        O1 = __builtin_amdgcn_mfma_f32_4x4x4f16(a1, b1, O1, 0, 0, 0);
                    } else {
#pragma unroll
                        for (int h = 0; h < kNH; h++) {
                            const h4 a0 = *reinterpret_cast<const h4 *>(pa0 + h * kPsH + tok);
                            const h4 a1 = *reinterpret_cast<const h4 *>(pa1 + h * kPsH + tok);
                            const h2 a00 = {a0[0], a0[1]}, a01 = {a0[2], a0[3]};
                            const h2 a10 = {a1[0], a1[1]}, a11 = {a1[2], a1[3]};
                            O0[h] = __builtin_amdgcn_fdot2(a00, x00, O0[h], false);
                            O0[h] = __builtin_amdgcn_fdot2(a01, x01, O0[h], false);
                            O1[h] = __builtin_amdgcn_fdot2(a10, x10, O1[h], false);
                            O1[h] = __builtin_amdgcn_fdot2(a11, x11, O1[h], false);
                        }
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // ---------------- finish the wave: undo operand scalings, add the zero-point term
    const float vun = 16777216.0f / 16.0f;                 // 2^24 (subnormal fields) / 2^4 (ps headroom)
    float lsum[kNH];
#pragma unroll
    for (int h = 0; h < kNH; h++) {
        lsum[h] = wave_sum64(l_lane[h]);
        float z0 = 0.f, z1 = 0.f;
#pragma unroll
        for (int g = 0; g < NCG; g++) {
            const float zs = wave_sum64(oz[h][g]);
            z0 = (g == cg0) ? zs : z0;
            z1 = (g == cg1) ? zs : z1;
        }
        O0[h] = O0[h] * vun + z0;
        O1[h] = O1[h] * vun + z1;
    }

    // ---------------- merge the four waves through LDS, write the split-K partial
    __syncthreads();
    float *mo = reinterpret_cast<float *>(lds);            // [4 waves][kNH][128]
    float *mm = mo + 4 * kNH * kD;                         // [4][kNH]
    float *ml = mm + 4 * kNH;
#pragma unroll
    for (int h = 0; h < kNH; h++) {
        mo[(wave * kNH + h) * kD + lane] = O0[h];
        mo[(wave * kNH + h) * kD + lane + 64] = O1[h];
        if (lane == 0) { mm[wave * kNH + h] = m[h]; ml[wave * kNH + h] = lsum[h]; }
    }
    __syncthreads();
    const int c = tid & 127;
    for (int h = tid >> 7; h < nheads; h += 2) {
        float M = -1e30f;
        for (int w = 0; w < 4; w++) M = fmaxf(M, mm[w * kNH + h]);
        float L = 0.f, O = 0.f;
        for (int w = 0; w < 4; w++) {
            const float sc = exp2f(mm[w * kNH + h] - M);
            L += ml[w * kNH + h] * sc;
            O += mo[(w * kNH + h) * kD + c] * sc;
        }
        float *pp = partial_ptr(a, bq0 + h, ch);
        pp[4 + c] = O;
        if (c == 0) { pp[0] = M; pp[1] = L; }
    }
}

template <int G, bool MFMA, bool LO>
static int launch_tiled(const DecArgs &a, int units, hipStream_t st)
{
    constexpr int NG = kPass / G > 0 ? kPass / G : 1;
    constexpr int NCG = kD / G;
    constexpr int WAVE_HALFS = (LO ? 2 : 1) * NG * kQsG + NCG * kPsG;
    constexpr size_t merge_bytes = (size_t)(4 * kNH * kD + 8 * kNH) * sizeof(float);
    constexpr size_t res_bytes = (size_t)kNH * kD * 2 + 4 * kNH * 64 * sizeof(float);
    size_t lds_bytes = (size_t)4 * WAVE_HALFS * 2;
    if (lds_bytes < merge_bytes) lds_bytes = merge_bytes;
    if (lds_bytes < res_bytes) lds_bytes = res_bytes;
    auto kern = decode_tiled_kernel<G, MFMA, LO>;
    static bool attr_set = false;                          // per instantiation
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_bytes) != hipSuccess)
            return MINIKV_ELAUNCH;
        attr_set = true;
    }
    dim3 grid(a.nchunk + 1, units, (a.rep + kNH - 1) / kNH);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds_bytes, st, a);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

template <bool MFMA>
static int launch_tiled_g(const DecArgs &a, int G, int units, hipStream_t st)
{
    switch (G) {
    case 16: return launch_tiled<16, MFMA, true>(a, units, st);
    case 32: return launch_tiled<32, MFMA, true>(a, units, st);
    case 64: return launch_tiled<64, MFMA, true>(a, units, st);
    case 128: return launch_tiled<128, MFMA, true>(a, units, st);
    }
    return MINIKV_EUNSUPPORTED;
}

int launch_decode_tiled(const DecArgs &a, int G, int units, bool mfma, hipStream_t st)
{
    return mfma ? launch_tiled_g<true>(a, G, units, st) : launch_tiled_g<false>(a, G, units, st);
}

}  // namespace minikv
