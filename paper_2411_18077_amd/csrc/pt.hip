// Per-token quantized KV cache: the token-wise quantization the paper's appendix studies (8, 4 and 2 bits for
// keys and values alike; 2 bits is the case it reports as failing) and its 4-bit baseline, whose size the
// appendix on KV cache compression ratios works out.  Keys are quantized like values: the G channels of one
// token share a zero-point and a scale.  Entry points: kv_quantize_pack_pt, minikv_decode_attn_pt.
//
// Storage (per unit; cpw = 32 / bits codes per word, code i of a word at bits [bits*i, bits*i + bits)):
//   Kc [Tcap][D/cpw]   token major (a token's codes are contiguous: the score phase has one token per thread)
//   Vc [Tcap/cpw][D]   channel major (a word = cpw consecutive tokens of one channel: the value phase has one
//                      channel per thread and consecutive threads read consecutive words)
//   Ks, Kz, Vs, Vz fp16 [Tcap][D/G];  q_len int32, a multiple of 16.
#include "common.h"

#include <hip/hip_fp16.h>

namespace minikv {

constexpr int kPtBlockTok = 64;      // tokens one workgroup of the quantizer takes
constexpr int kPtSB = 256;           // tokens per inner block of the decode kernel (= threads)
constexpr int kPtMaxRep = 8;

struct PtQuantArgs {
    const uint16_t *K, *V;
    const int32_t *idx, *n_tok;
    uint32_t *Kc, *Vc;
    uint16_t *Ks, *Kz, *Vs, *Vz;
    int32_t *q_len;
    int64_t L, idx_stride;
    int Tcap, max_tok;
};

__device__ inline float pt_h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// Tokens this unit appends, or 0 when the request is not a positive multiple of 16 that fits.
__device__ inline int pt_tokens_to_append(const PtQuantArgs &a, int u, int &q0)
{
    const int n = a.n_tok[u];
    q0 = a.q_len[u];
    if (n <= 0 || (n & 15) || q0 < 0 || (q0 & 15) || q0 + n > a.Tcap || n > a.L || n > a.max_tok) return 0;
    return n;
}

// The quantizer of one group: zero = min (fp16, -0 stored as +0), scale = fp16((max - min) / levels) in
// binary32, 1/scale of the STORED scale; every operation separately rounded (this file is compiled without
// floating-point contraction).
__device__ inline void pt_group_params(float mn, float mx, float levels, uint16_t &sh, uint16_t &zh, float &inv, float &zf)
{
    zh = __half_as_ushort(__float2half_rn(mn));
    if ((zh & 0x7fffu) == 0) zh = 0;
    zf = pt_h2f(zh);
    const float range = mx - mn;
    const float step = range / levels;
    const __half s = __float2half_rn(step);
    sh = __half_as_ushort(s);
    const float sf = __half2float(s);
    inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
}
__device__ inline uint32_t pt_code(float x, float zf, float inv, float levels)
{
    const float d = x - zf;
    const float u = d * inv;
    return (uint32_t)(int)__builtin_amdgcn_fmed3f(rintf(u), 0.0f, levels);
}

// One thread = 16 consecutive channels of one token; a group of G channels = G/16 neighbouring threads.
// Returns the thread's 16 codes; the group's first thread stores scale and zero-point at meta_at.
template <int BITS, int G>
__device__ inline void pt_quantize_slice(const uint16_t *row16, uint16_t *sc, uint16_t *zp, int slice, uint32_t (&codes)[16])
{
    constexpr float levels = (float)((1 << BITS) - 1);
    const uint4 a = reinterpret_cast<const uint4 *>(row16)[0], b = reinterpret_cast<const uint4 *>(row16)[1];
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    float x[16];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        x[2 * i] = pt_h2f((uint16_t)(w[i] & 0xffffu));
        x[2 * i + 1] = pt_h2f((uint16_t)(w[i] >> 16));
    }
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int i = 1; i < 16; i++) { mn = fminf(mn, x[i]); mx = fmaxf(mx, x[i]); }
#pragma unroll
    for (int d = 1; d < G / 16; d <<= 1) {           // the G/16 threads of the group are neighbours in the wave
        mn = fminf(mn, __shfl_xor(mn, d));
        mx = fmaxf(mx, __shfl_xor(mx, d));
    }
    uint16_t sh, zh;
    float inv, zf;
    pt_group_params(mn, mx, levels, sh, zh, inv, zf);
    if ((slice & (G / 16 - 1)) == 0) { sc[slice / (G / 16)] = sh; zp[slice / (G / 16)] = zh; }
#pragma unroll
    for (int i = 0; i < 16; i++) codes[i] = pt_code(x[i], zf, inv, levels);
}

template <int BITS, int G>
__global__ __launch_bounds__(256) void quantize_pack_pt_kernel(PtQuantArgs a)
{
    constexpr int CPW = 32 / BITS, NG = kD / G;
    __shared__ uint8_t vcode[kPtBlockTok][kD + 4];     // V codes of the block, one byte each (row pitch 132)

    const int u = blockIdx.y, tid = threadIdx.x;
    int q0;
    const int n = pt_tokens_to_append(a, u, q0);
    const int i0 = blockIdx.x * kPtBlockTok;
    if (i0 >= n) return;
    const int nt = min(kPtBlockTok, n - i0);           // multiple of 16
    const int t0 = q0 + i0;

    const int slice = tid & 7;                         // 16-channel slice of the token
    for (int i = tid >> 3; i < nt; i += 32) {
        long row = a.idx ? (long)a.idx[(size_t)u * a.idx_stride + i0 + i] : (long)(i0 + i);
        row = row < 0 ? 0 : (row >= a.L ? a.L - 1 : row);
        const size_t src = ((size_t)u * a.L + row) * kD + slice * 16;
        const size_t meta = ((size_t)u * a.Tcap + (size_t)(t0 + i)) * NG;
        uint32_t codes[16];
        // keys: the codes of a token are contiguous, 16 codes = 16 * BITS / 32 words
        pt_quantize_slice<BITS, G>(a.K + src, a.Ks + meta, a.Kz + meta, slice, codes);
        uint32_t *kdst = a.Kc + ((size_t)u * a.Tcap + (size_t)(t0 + i)) * (kD / CPW) + slice * (16 / CPW);
#pragma unroll
        for (int wv = 0; wv < 16 / CPW; wv++) {
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < CPW; j++) word |= codes[wv * CPW + j] << (BITS * j);
            kdst[wv] = word;
        }
        // values: codes go through LDS, the words run along the tokens
        pt_quantize_slice<BITS, G>(a.V + src, a.Vs + meta, a.Vz + meta, slice, codes);
#pragma unroll
        for (int j = 0; j < 16; j++) vcode[i][slice * 16 + j] = (uint8_t)codes[j];
    }
    __syncthreads();
    uint32_t *vdst = a.Vc + (size_t)u * (size_t)(a.Tcap / CPW) * kD + (size_t)(t0 / CPW) * kD;
    for (int wi = tid; wi < (nt / CPW) * kD; wi += 256) {
        const int r = wi / kD, c = wi % kD;
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < CPW; j++) word |= (uint32_t)vcode[r * CPW + j][c] << (BITS * j);
        vdst[(size_t)r * kD + c] = word;
    }
}

__global__ void update_lengths_pt_kernel(PtQuantArgs a, int units)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    int q0;
    const int n = pt_tokens_to_append(a, u, q0);
    if (n) a.q_len[u] = q0 + n;
}

// ------------------------------------------------------------------------------------------------ decode
struct PtDecArgs {
    const uint16_t *q;
    const uint32_t *Kc, *Vc;
    const uint16_t *Ks, *Kz, *Vs, *Vz;
    const int32_t *q_len;
    uint16_t *out;
    float *ws;                    // partials [B*Hq][nchunk][kPartialStride]: m, l, 2 pad, o[128]
    float c1;                     // sm_scale * log2(e)
    int Hq, Hkv, rep, Tcap, chunk, nchunk;
};

__device__ inline float pt_wave_max(float v)
{
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float pt_wave_sum(float v)
{
    for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// A 16-bit half of a packed word holds NF = 16 / BITS codes.  A code field that lies inside bits 0..9 of its
// half is, masked in place, an fp16 SUBNORMAL: code * 2^(BITS*pos) * 2^-24 -- so one v_and_b32 "converts" two
// codes (one per half) and one v_dot2_f32_f16 multiplies them with two fp16 operands and adds both products
// in binary32 (fp16 subnormals are honoured by that instruction).  Fields at positions 0 .. PMAX-1 are taken
// from the word as it is, the others from the word shifted right by SH2 bits, which brings them to positions
// NF-PMAX .. PMAX-1 ... of a field j: pt_field_pos().  Sums are kept per position and scaled once at the end.
template <int BITS> struct PtFields {
    static constexpr int NF = 16 / BITS;                 // fields per half-word
    static constexpr int PMAX = 10 / BITS;               // positions whose field fits into the fp16 mantissa
    static constexpr int SH2 = BITS * (NF - PMAX);       // shift that brings the upper fields down
    static constexpr uint32_t M0 = ((1u << BITS) - 1u) * 0x00010001u;
    static_assert(NF <= 2 * PMAX, "two looks at a word reach every field");
    __device__ static constexpr int pos(int j) { return j < PMAX ? j : j - (NF - PMAX); }
    // 2^(24 - BITS*pos): what a sum over position pos is multiplied by
    __device__ static constexpr float unscale(int p) { return 16777216.0f / (float)(1u << (BITS * p)); }
};
typedef _Float16 pt_h2 __attribute__((ext_vector_type(2)));

// One workgroup = one (unit, chunk of tokens), all query heads of the unit.  Per inner block of 256 tokens:
// score phase, one token per thread -- sum_c q_c * (code * Ks + Kz) = sum_g Ks_g * (sum_{c in g} q_c code_c)
// + Kz_g * (sum_{c in g} q_c), so the codes meet the query before any scale does; the query sits in LDS as
// the fp16 pairs (channel c0 + j, channel c0 + NF + j) that the two halves of a word's field j hold --;
// block-wide online softmax; value phase, one channel per thread, the weights times the token's V scale in LDS
// as fp16 pairs (token t0 + j, token t0 + NF + j) in the same way; the zero-point term kept per token thread
// and reduced once at the end.
template <int BITS, int G, int REPT>
__global__ __launch_bounds__(256, 2) void decode_pt_kernel(PtDecArgs a)
{
    typedef PtFields<BITS> F;
    constexpr int CPW = 32 / BITS, NG = kD / G, W = kD / CPW, NF = F::NF, NP = F::PMAX;
    constexpr int NPAIR = kPtSB / 2;                                     // weight pairs of a block
    __shared__ float qsum[REPT][NG];                                     // sums of q over the channel groups
    __shared__ __attribute__((aligned(16))) pt_h2 qp[kD / 2][REPT];      // query pairs, by (word, field)
    __shared__ __attribute__((aligned(16))) pt_h2 wp[NG][NPAIR][REPT];   // weight * V scale pairs, by (word, field)
    __shared__ float red[4][REPT];
    __shared__ float comb[REPT][kD];
    __shared__ float zsum[REPT][NG];

    const int u = blockIdx.y, ch = blockIdx.x, tid = threadIdx.x, rep = a.rep;
    const int b = u / a.Hkv, kvh = u % a.Hkv;
    const int bq0 = b * a.Hq + kvh * rep;
    const int T = min(max(a.q_len[u], 0), a.Tcap);
    const int t_begin = ch * a.chunk, t_end = min(T, t_begin + a.chunk);
    if (t_begin >= t_end) return;                       // the merge kernel skips this slot

    // heads beyond rep read the unit's last head and are never written out
    for (int i = tid; i < (kD / 2) * REPT; i += 256) {
        const int h = i % REPT, pi = i / REPT, w = pi / NF, j = pi % NF;
        const uint16_t *qr = a.q + (size_t)(bq0 + min(h, rep - 1)) * kD + w * CPW + j;
        pt_h2 v;
        v[0] = __builtin_bit_cast(_Float16, qr[0]);
        v[1] = __builtin_bit_cast(_Float16, qr[NF]);
        qp[pi][h] = v;
    }
    if (tid < REPT * NG) {
        const int h = tid / NG, g = tid % NG;
        float s = 0.f;
        for (int c = 0; c < G; c++) s += pt_h2f(a.q[(size_t)(bq0 + min(h, rep - 1)) * kD + g * G + c]);
        qsum[h][g] = s;
    }
    __syncthreads();

    const uint32_t *Kc = a.Kc + (size_t)u * a.Tcap * W;
    const uint32_t *Vc = a.Vc + (size_t)u * (size_t)(a.Tcap / CPW) * kD;
    const uint16_t *Ks = a.Ks + (size_t)u * a.Tcap * NG, *Kz = a.Kz + (size_t)u * a.Tcap * NG;
    const uint16_t *Vs = a.Vs + (size_t)u * a.Tcap * NG, *Vz = a.Vz + (size_t)u * a.Tcap * NG;

    float m[REPT], l[REPT], o[REPT], pz[REPT][NG];
#pragma unroll
    for (int h = 0; h < REPT; h++) {
        m[h] = -1e30f; l[h] = 0.f; o[h] = 0.f;
#pragma unroll
        for (int g = 0; g < NG; g++) pz[h][g] = 0.f;
    }
    const int c = tid & (kD - 1), half = tid >> 7, cg = c / G;
    // where this thread's token puts its weight: pair (tid / CPW) * NF + (tid % CPW) % NF, component (tid % CPW) / NF
    const int my_pair = (tid / CPW) * NF + (tid % CPW) % NF, my_comp = (tid % CPW) / NF;

    // The words of a block are requested well before they are used: the key words, scales and zero-points
    // of the NEXT block right after the score phase has consumed this block's, the value words of this
    // block before its score phase.  (A load that waits for its predecessor's data costs a full memory
    // round trip; sixteen of those per block is what bounds a version without this.)
    constexpr int NVW = 128 / CPW;                      // value words of one thread and block
    uint4 kq[W / 4];
    uint16_t ksr[NG], kzr[NG], vsr[NG], vzr[NG];
    auto request_k = [&](int ts_) {
        const int tc_ = min(ts_ + tid, t_end - 1);
        const uint4 *kw4 = reinterpret_cast<const uint4 *>(Kc + (size_t)tc_ * W);
#pragma unroll
        for (int i = 0; i < W / 4; i++) kq[i] = kw4[i];
#pragma unroll
        for (int g = 0; g < NG; g++) {
            ksr[g] = Ks[(size_t)tc_ * NG + g]; kzr[g] = Kz[(size_t)tc_ * NG + g];
            vsr[g] = Vs[(size_t)tc_ * NG + g]; vzr[g] = Vz[(size_t)tc_ * NG + g];
        }
    };
    request_k(t_begin);
    const int vrow_last = a.Tcap / CPW - 1;

    // sums over the field positions, each with its power of two
    auto fold = [&](const float (&acc)[NP]) -> float {
        float r = 0.f;
#pragma unroll
        for (int p = 0; p < NP; p++) r = __builtin_fmaf(acc[p], F::unscale(p), r);
        return r;
    };

    for (int ts = t_begin; ts < t_end; ts += kPtSB) {
        const bool valid = ts + tid < t_end;
        // (an index the compiler cannot see through: without it the reads of the query pairs, which no iteration
        // changes, are all moved in front of the loop and held in 64 x REPT registers)
        int iter0 = 0;
        asm volatile("" : "+v"(iter0));
        uint32_t vw[NVW];                               // rows past the cache's end repeat its last row: their weights are 0
#pragma unroll
        for (int i = 0; i < NVW; i++) vw[i] = Vc[(size_t)min((ts + half * 128) / CPW + i, vrow_last) * kD + c];
        __builtin_amdgcn_sched_barrier(0);
        // ---- scores of token ts + tid
        float s[REPT];
#pragma unroll
        for (int h = 0; h < REPT; h++) s[h] = 0.f;
        float vs[NG], vz[NG];
        {
            // the query pairs of one word at a time (scheduling barriers keep it so: left alone, the compiler
            // requests all 64 x REPT pairs at once and spills); the other waves of the SIMD cover the LDS latency
            // The query pairs of word wi + 1 are read from LDS while the products of word wi run.  Left alone, the
            // compiler requests the pairs of all 64 words first and spills what comes back (scheduling barriers and
            // plain memory barriers do not stop it: the products have no side effects and sink below them); so each
            // word ends with empty asm statements that take its sums as operands AND clobber memory: the next
            // reads cannot pass them, and they cannot pass the products.
            pt_h2 qa[NF][REPT], qb[NF][REPT];
            auto read_q = [&](pt_h2 (&dst)[NF][REPT], int wi) {
#pragma unroll
                for (int j = 0; j < NF; j++)
#pragma unroll
                    for (int h = 0; h < REPT; h++) dst[j][h] = qp[iter0 + wi * NF + j][h];
            };
            read_q(qa, 0);
            float dot[REPT][NP];
#pragma unroll
            for (int wi = 0; wi < W; wi++) {
                constexpr int WG_ = G / CPW;                                   // words of one channel group
                const int g = wi / WG_;
                if (wi % WG_ == 0) {
#pragma unroll
                    for (int h = 0; h < REPT; h++)
#pragma unroll
                        for (int p = 0; p < NP; p++) dot[h][p] = 0.f;
                }
                if (wi + 1 < W) read_q(qb, wi + 1);
                const uint4 q4 = kq[wi / 4];
                const uint32_t word = (wi & 3) == 0 ? q4.x : (wi & 3) == 1 ? q4.y : (wi & 3) == 2 ? q4.z : q4.w;
                const uint32_t upper = word >> F::SH2;
#pragma unroll
                for (int j = 0; j < NF; j++) {
                    const int p = F::pos(j);
                    const uint32_t fld = (j < F::PMAX ? word : upper) & (F::M0 << (BITS * p));
                    const pt_h2 kk = __builtin_bit_cast(pt_h2, fld);
#pragma unroll
                    for (int h = 0; h < REPT; h++) dot[h][p] = __builtin_amdgcn_fdot2(kk, qa[j][h], dot[h][p], false);
                }
#pragma unroll
                for (int h = 0; h < REPT; h++)
#pragma unroll
                    for (int p = 0; p < NP; p++) asm volatile("" : "+v"(dot[h][p])::"memory");
                if (wi % WG_ == WG_ - 1) {                                     // the group's last word: its scale and zero-point
                    const float ks = pt_h2f(ksr[g]), kz = pt_h2f(kzr[g]);
                    vs[g] = pt_h2f(vsr[g]); vz[g] = pt_h2f(vzr[g]);
#pragma unroll
                    for (int h = 0; h < REPT; h++) s[h] += ks * fold(dot[h]) + kz * qsum[h][g];
                }
#pragma unroll
                for (int j = 0; j < NF; j++)
#pragma unroll
                    for (int h = 0; h < REPT; h++) qa[j][h] = qb[j][h];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (ts + kPtSB < t_end) request_k(ts + kPtSB);
        __builtin_amdgcn_sched_barrier(0);
        // ---- block max, weights, block sum
#pragma unroll
        for (int h = 0; h < REPT; h++) {
            s[h] = valid ? s[h] * a.c1 : -INFINITY;       // base-2 domain
            const float wm = pt_wave_max(s[h]);
            if ((tid & 63) == 0) red[tid >> 6][h] = wm;
        }
        __syncthreads();
        float scale[REPT], p[REPT];
#pragma unroll
        for (int h = 0; h < REPT; h++) {
            const float bm = fmaxf(fmaxf(red[0][h], red[1][h]), fmaxf(red[2][h], red[3][h]));
            const float mn = fmaxf(m[h], bm);
            scale[h] = exp2f(m[h] - mn);
            m[h] = mn;
            p[h] = exp2f(s[h] - mn);                    // exp2(-inf) = 0 for the masked tail
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < REPT; h++) {
            // (the value phase sees p * Vs rounded to fp16; the sum of weights keeps the binary32 p)
            const float ws = pt_wave_sum(p[h]);
            if ((tid & 63) == 0) red[tid >> 6][h] = ws;
#pragma unroll
            for (int g = 0; g < NG; g++) {
                reinterpret_cast<_Float16 *>(&wp[g][my_pair][h])[my_comp] = (_Float16)(p[h] * vs[g]);
                pz[h][g] = pz[h][g] * scale[h] + p[h] * vz[g];
            }
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < REPT; h++) {
            l[h] = l[h] * scale[h] + (red[0][h] + red[1][h] + red[2][h] + red[3][h]);
            o[h] *= scale[h];
        }
        // ---- weighted values: thread (c, half) takes tokens [half*128, half*128 + 128) of the block
        float oacc[REPT][NP];
#pragma unroll
        for (int h = 0; h < REPT; h++)
#pragma unroll
            for (int pp = 0; pp < NP; pp++) oacc[h][pp] = 0.f;
        {
            pt_h2 wa[NF][REPT], wb[NF][REPT];                                   // weight pairs of word i, word i + 1
            auto read_w = [&](pt_h2 (&dst)[NF][REPT], int i) {
#pragma unroll
                for (int j = 0; j < NF; j++)
#pragma unroll
                    for (int h = 0; h < REPT; h++) dst[j][h] = wp[cg][iter0 + ((half * 128) / CPW + i) * NF + j][h];
            };
            read_w(wa, 0);
#pragma unroll
            for (int i = 0; i < NVW; i++) {
                // (words past the block's last token meet weights that are 0: no branch)
                if (i + 1 < NVW) read_w(wb, i + 1);
                const uint32_t word = vw[i], upper = word >> F::SH2;
#pragma unroll
                for (int j = 0; j < NF; j++) {
                    const int pp = F::pos(j);
                    const uint32_t fld = (j < F::PMAX ? word : upper) & (F::M0 << (BITS * pp));
                    const pt_h2 vv = __builtin_bit_cast(pt_h2, fld);
#pragma unroll
                    for (int h = 0; h < REPT; h++) oacc[h][pp] = __builtin_amdgcn_fdot2(vv, wa[j][h], oacc[h][pp], false);
                }
#pragma unroll
                for (int h = 0; h < REPT; h++)
#pragma unroll
                    for (int pp = 0; pp < NP; pp++) asm volatile("" : "+v"(oacc[h][pp])::"memory");
#pragma unroll
                for (int j = 0; j < NF; j++)
#pragma unroll
                    for (int h = 0; h < REPT; h++) wa[j][h] = wb[j][h];
            }
        }
#pragma unroll
        for (int h = 0; h < REPT; h++) o[h] += fold(oacc[h]);
        __syncthreads();
    }

    // ---- zero-point term: sum over the token threads, per (head, channel group)
    if (tid < REPT * NG) zsum[tid / NG][tid % NG] = 0.f;
    __syncthreads();
#pragma unroll
    for (int h = 0; h < REPT; h++) {
#pragma unroll
        for (int g = 0; g < NG; g++) {
            const float wsum = pt_wave_sum(pz[h][g]);
            if ((tid & 63) == 0) atomicAdd(&zsum[h][g], wsum);
        }
    }
    if (half == 1) {
#pragma unroll
        for (int h = 0; h < REPT; h++) comb[h][c] = o[h];
    }
    __syncthreads();
    if (half == 0) {
#pragma unroll
        for (int h = 0; h < REPT; h++) {
            if (h < rep) {
                float *pp = a.ws + ((size_t)(bq0 + h) * a.nchunk + ch) * kPartialStride;
                pp[4 + c] = o[h] + comb[h][c] + zsum[h][cg];
                if (c == 0) { pp[0] = m[h]; pp[1] = l[h]; }
            }
        }
    }
}

// One workgroup of 128 threads per query row: combine the partials of the chunks that hold tokens.  Eight
// chunks at a time, all their loads requested before the first is used; the running maximum is carried from
// batch to batch (online, like the kernel above).
__global__ __launch_bounds__(128) void merge_pt_kernel(PtDecArgs a)
{
    const int bq = blockIdx.x, c = threadIdx.x;
    const int u = (bq / a.Hq) * a.Hkv + (bq % a.Hq) / a.rep;
    const float *base = a.ws + (size_t)bq * a.nchunk * kPartialStride;
    float pm[8], pl[8], po[8];
    // (the first batch is requested before the unit's length is known: slots beyond it are ignored below)
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const float *p = base + (size_t)min(j, a.nchunk - 1) * kPartialStride;
        pm[j] = p[0], pl[j] = p[1], po[j] = p[4 + c];
    }
    const int T = min(max(a.q_len[u], 0), a.Tcap);
    const int nq = (T + a.chunk - 1) / a.chunk;
    float M = -1e30f, L = 0.f, O = 0.f;
    for (int c0 = 0; c0 < nq; c0 += 8) {
        if (c0) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const float *p = base + (size_t)min(c0 + j, nq - 1) * kPartialStride;
                pm[j] = p[0], pl[j] = p[1], po[j] = p[4 + c];
            }
        }
        float bm = M;
#pragma unroll
        for (int j = 0; j < 8; j++) bm = c0 + j < nq ? fmaxf(bm, pm[j]) : bm;
        const float sc = exp2f(M - bm);
        L *= sc, O *= sc, M = bm;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const bool in = c0 + j < nq;                   // (a slot beyond the unit's chunks holds anything, NaN included)
            const float w = exp2f(pm[j] - M);
            L = in ? __builtin_fmaf(pl[j], w, L) : L;
            O = in ? __builtin_fmaf(po[j], w, O) : O;
        }
    }
    a.out[(size_t)bq * kD + c] = __half_as_ushort(__float2half_rn(L > 0.f ? O / L : 0.f));
}

static int pt_validate_shape(const minikv_pt_shape *s)
{
    if (!s) return MINIKV_EINVAL;
    if (s->D != kD) return MINIKV_EUNSUPPORTED;
    if (!(s->G == 32 || s->G == 64 || s->G == 128)) return MINIKV_EUNSUPPORTED;
    if (!(s->bits == 2 || s->bits == 4 || s->bits == 8)) return MINIKV_EUNSUPPORTED;
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv) return MINIKV_EINVAL;
    if (s->Hq / s->Hkv > kPtMaxRep) return MINIKV_EUNSUPPORTED;
    if (s->Tcap <= 0 || s->Tcap % 64) return MINIKV_EINVAL;
    if ((int64_t)s->B * s->Hkv > 65535) return MINIKV_EINVAL;
    return MINIKV_OK;
}

static int pt_validate_cache(const minikv_pt_cache *c)
{
    if (!c) return MINIKV_EINVAL;
    if (!aligned16(c->Kc) || !aligned16(c->Ks) || !aligned16(c->Kz) || !aligned16(c->Vc) || !aligned16(c->Vs) ||
        !aligned16(c->Vz) || !c->q_len)
        return MINIKV_EINVAL;
    return MINIKV_OK;
}

// token chunk of one decode workgroup: a multiple of the 256-token block, as long as the launch keeps more
// than a thousand workgroups (a workgroup sets up the query pairs once, so chunks of several blocks pay;
// chunks of one block measured 5-20 % slower on the batch-32 configuration)
static int pt_chunk(const minikv_pt_shape &s)
{
    const long units = (long)s.B * s.Hkv;
    int chunk = kPtSB;
    while (chunk < 8192 && units * ((s.Tcap + 2 * chunk - 1) / (2 * chunk)) >= 1024) chunk *= 2;
    return chunk;
}

template <int BITS>
static int pt_launch_quantize(const PtQuantArgs &a, int G, dim3 grid, int units, hipStream_t st)
{
    switch (G) {
    case 32: hipLaunchKernelGGL((quantize_pack_pt_kernel<BITS, 32>), grid, dim3(256), 0, st, a); break;
    case 64: hipLaunchKernelGGL((quantize_pack_pt_kernel<BITS, 64>), grid, dim3(256), 0, st, a); break;
    case 128: hipLaunchKernelGGL((quantize_pack_pt_kernel<BITS, 128>), grid, dim3(256), 0, st, a); break;
    default: return MINIKV_EUNSUPPORTED;
    }
    hipLaunchKernelGGL(update_lengths_pt_kernel, dim3((units + 255) / 256), dim3(256), 0, st, a, units);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

template <int BITS, int REPT>
static int pt_launch_decode_g(const PtDecArgs &a, int G, dim3 grid, hipStream_t st)
{
    switch (G) {
    case 32: hipLaunchKernelGGL((decode_pt_kernel<BITS, 32, REPT>), grid, dim3(256), 0, st, a); break;
    case 64: hipLaunchKernelGGL((decode_pt_kernel<BITS, 64, REPT>), grid, dim3(256), 0, st, a); break;
    case 128: hipLaunchKernelGGL((decode_pt_kernel<BITS, 128, REPT>), grid, dim3(256), 0, st, a); break;
    default: return MINIKV_EUNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

// heads per unit rounded up to 1, 2, 4 or 8 (the spare ones repeat the last head and are not written)
template <int BITS>
static int pt_launch_decode(const PtDecArgs &a, int G, dim3 grid, hipStream_t st)
{
    if (a.rep <= 1) return pt_launch_decode_g<BITS, 1>(a, G, grid, st);
    if (a.rep <= 2) return pt_launch_decode_g<BITS, 2>(a, G, grid, st);
    if (a.rep <= 4) return pt_launch_decode_g<BITS, 4>(a, G, grid, st);
    return pt_launch_decode_g<BITS, 8>(a, G, grid, st);
}

}  // namespace minikv

using namespace minikv;

extern "C" {

size_t minikv_pt_cache_bytes(const minikv_pt_shape *s, int which)
{
    if (pt_validate_shape(s) != MINIKV_OK) return 0;
    const size_t U = (size_t)s->B * s->Hkv;
    switch (which) {
    case MINIKV_BUF_KC:
    case MINIKV_BUF_VC: return U * (size_t)s->Tcap * (size_t)(kD * s->bits / 8);
    case MINIKV_BUF_KS:
    case MINIKV_BUF_KZ:
    case MINIKV_BUF_VS:
    case MINIKV_BUF_VZ: return U * (size_t)s->Tcap * (size_t)(kD / s->G) * 2;
    case MINIKV_BUF_QLEN: return U * 4;
    default: return 0;
    }
}

size_t minikv_pt_workspace_bytes(const minikv_pt_shape *s)
{
    if (pt_validate_shape(s) != MINIKV_OK) return 0;
    const int chunk = pt_chunk(*s);
    const size_t nchunk = (size_t)(s->Tcap + chunk - 1) / chunk;
    return (size_t)s->B * s->Hq * nchunk * kPartialStride * sizeof(float);
}

int kv_quantize_pack_pt(const minikv_pt_shape *s, const minikv_f16 *K, const minikv_f16 *V, int64_t L,
                        const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, int32_t max_tok,
                        minikv_pt_cache *c, void *stream)
{
    int rc = pt_validate_shape(s);
    if (rc) return rc;
    if ((rc = pt_validate_cache(c))) return rc;
    if (!aligned16(K) || !aligned16(V) || !n_tok || L <= 0) return MINIKV_EINVAL;
    if (max_tok < 0 || max_tok % 16 || max_tok > s->Tcap || max_tok > L) return MINIKV_EINVAL;
    if (idx && idx_stride < max_tok) return MINIKV_EINVAL;
    if (max_tok == 0) return MINIKV_OK;
    PtQuantArgs a;
    a.K = K; a.V = V; a.idx = idx; a.n_tok = n_tok;
    a.Kc = c->Kc; a.Vc = c->Vc; a.Ks = c->Ks; a.Kz = c->Kz; a.Vs = c->Vs; a.Vz = c->Vz; a.q_len = c->q_len;
    a.L = L; a.idx_stride = idx_stride; a.Tcap = s->Tcap; a.max_tok = max_tok;
    const int units = s->B * s->Hkv;
    const dim3 grid((max_tok + kPtBlockTok - 1) / kPtBlockTok, units);
    switch (s->bits) {
    case 2: return pt_launch_quantize<2>(a, s->G, grid, units, (hipStream_t)stream);
    case 4: return pt_launch_quantize<4>(a, s->G, grid, units, (hipStream_t)stream);
    case 8: return pt_launch_quantize<8>(a, s->G, grid, units, (hipStream_t)stream);
    }
    return MINIKV_EUNSUPPORTED;
}

int minikv_decode_attn_pt(const minikv_pt_shape *s, const minikv_f16 *q, const minikv_pt_cache *c, float sm_scale,
                          minikv_f16 *out, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = pt_validate_shape(s);
    if (rc) return rc;
    if ((rc = pt_validate_cache(c))) return rc;
    if (!aligned16(q) || !aligned16(out) || !aligned16(workspace)) return MINIKV_EINVAL;
    if (!(sm_scale == sm_scale) || sm_scale - sm_scale != 0.0f) return MINIKV_EINVAL;
    if (workspace_bytes < minikv_pt_workspace_bytes(s)) return MINIKV_EWORKSPACE;
    PtDecArgs a;
    a.q = q; a.Kc = c->Kc; a.Vc = c->Vc; a.Ks = c->Ks; a.Kz = c->Kz; a.Vs = c->Vs; a.Vz = c->Vz; a.q_len = c->q_len;
    a.out = out;
    a.ws = reinterpret_cast<float *>(workspace);
    a.c1 = sm_scale * 1.44269504088896340736f;
    a.Hq = s->Hq; a.Hkv = s->Hkv; a.rep = s->Hq / s->Hkv; a.Tcap = s->Tcap;
    a.chunk = pt_chunk(*s);
    a.nchunk = (s->Tcap + a.chunk - 1) / a.chunk;
    const dim3 grid(a.nchunk, s->B * s->Hkv);
    switch (s->bits) {
    case 2: rc = pt_launch_decode<2>(a, s->G, grid, (hipStream_t)stream); break;
    case 4: rc = pt_launch_decode<4>(a, s->G, grid, (hipStream_t)stream); break;
    case 8: rc = pt_launch_decode<8>(a, s->G, grid, (hipStream_t)stream); break;
    default: return MINIKV_EUNSUPPORTED;
    }
    if (rc) return rc;
    hipLaunchKernelGGL(merge_pt_kernel, dim3(s->B * s->Hq), dim3(128), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

}  // extern "C"
