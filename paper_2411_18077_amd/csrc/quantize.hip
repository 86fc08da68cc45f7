// kv_quantize_pack / kv_flush_residual / kv_append_residual kernels (gfx950).
//
// Quantizer: Section 3.1.1 and Section 3.3 of the MiniKV paper -- asymmetric 2-bit codes, K grouped
// along tokens per channel, V grouped along channels per token, fp16 scale and zero-point, 16 codes per
// 32-bit word.  Residual buffer: Algorithm 1 lines 9-15.
//
// One workgroup of 256 threads takes a block of BT = max(64, G) consecutive retained tokens of one unit:
// the fp16 rows are gathered (Algorithm 1 line 3: only retained rows are read) into LDS with 128-bit
// loads, group statistics are taken from LDS, and each thread then builds whole 32-bit words so that
// every store is a full word and consecutive threads write consecutive addresses.
#include "common.h"

#include <hip/hip_fp16.h>

#include <type_traits>

namespace minikv {

struct QuantArgs {
    const uint16_t *K, *V;       // [U][L][D] fp16
    const int32_t *idx;          // [U][idx_stride] or null
    const int32_t *n_tok;        // [U]  (flush: r_len)
    uint32_t *Kc, *Vc;
    uint16_t *Ks, *Kz, *Vs, *Vz;
    int32_t *q_len, *r_len;
    int64_t L, idx_stride;
    int Tcap, Rcap, flush;
    int max_tok;                 // host-side bound of n_tok the launch was sized for
};

constexpr int kRow = kD + 8;     // LDS row pitch in halfs: 272 B keeps 16-B alignment, staggers banks

__device__ inline float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// Tokens this unit appends, or 0 when the request is not a positive multiple of G that fits.
template <int G>
__device__ inline int tokens_to_append(const QuantArgs &a, int u, int &q0)
{
    int n = a.n_tok[u];
    q0 = a.q_len[u];
    if (a.flush) n = (n == a.Rcap) ? a.Rcap : 0;
    if (n <= 0 || (n % G) || q0 < 0 || (q0 % G) || q0 + n > a.Tcap || n > a.L || n > a.max_tok) return 0;
    return n;
}

// scale (fp16 bits), zero (fp16 bits), 1/scale (binary32) of a group with extrema mn, mx.
__device__ inline void group_params(float mn, float mx, uint16_t &sh, uint16_t &zh, float &inv, float &zf)
{
    __half z = __float2half_rn(mn);                   // exact: mn is an fp16 value
    zh = __half_as_ushort(z);
    if ((zh & 0x7fffu) == 0) zh = 0;                  // -0 is stored as +0
    zf = h2f(zh);
    float range = mx - mn;
    float step = range / 3.0f;                        // IEEE binary32 division
    __half s = __float2half_rn(step);
    sh = __half_as_ushort(s);
    float sf = __half2float(s);
    inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
}

__device__ inline uint32_t quant_code(float x, float zf, float inv)
{
    float d = x - zf;
    float u = d * inv;
    float r = rintf(u);                               // round half to even
    r = fminf(fmaxf(r, 0.0f), 3.0f);
    return (uint32_t)(int)r;
}

// Where the rows this thread gathers start (in halfs from the tensor's base): the same for K and for V, so the
// positions are read, clamped and turned into offsets once.  Thread t moves the 16-byte piece t % 16 of rows
// t / 16, t / 16 + 16, ...
template <int NR>
__device__ __forceinline__ void row_offsets(size_t (&off)[NR], const QuantArgs &a, int u, int i0, int nt)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < NR; j++) {
        const int r = (tid >> 4) + 16 * j;
        long row = 0;
        if (r < nt) row = a.idx ? (long)a.idx[(size_t)u * a.idx_stride + i0 + r] : (long)(i0 + r);
        row = row < 0 ? 0 : (row >= a.L ? a.L - 1 : row);
        off[j] = ((size_t)u * a.L + row) * kD + (tid & 15) * 8;
    }
}
template <int NR>
__device__ __forceinline__ void load_rows(uint16_t *tile, const uint16_t *src, const size_t (&off)[NR], int nt)
{
    const int tid = threadIdx.x;
    uint4 x[NR];                                       // (rows past the block read row 0 of the unit and are not stored)
#pragma unroll
    for (int j = 0; j < NR; j++) x[j] = *reinterpret_cast<const uint4 *>(src + off[j]);
#pragma unroll
    for (int j = 0; j < NR; j++)
        if ((tid >> 4) + 16 * j < nt) *reinterpret_cast<uint4 *>(tile + ((tid >> 4) + 16 * j) * kRow + (tid & 15) * 8) = x[j];
}

typedef _Float16 qh2 __attribute__((ext_vector_type(2)));
__device__ inline qh2 as_qh2(uint32_t u) { return __builtin_bit_cast(qh2, u); }
__device__ inline qh2 pk_min(qh2 a, qh2 b) { return __builtin_elementwise_min(a, b); }
__device__ inline qh2 pk_max(qh2 a, qh2 b) { return __builtin_elementwise_max(a, b); }

// code of x as a float 0..3 (round half to even, clamped): every operation a separately rounded binary32 one.
// nzi = (-zero, 1/scale).  x - zero is written as the fused x * one + (-zero) with `one` a 1.0 the compiler cannot
// see through: the conversion of the fp16 x then folds into the instruction (v_fma_mix_f32) and the result is
// the same single rounding of x - zero.
__device__ inline float quant_codef(_Float16 x, float2 nzi, float one)
{
    const float d = __builtin_fmaf((float)x, one, nzi.x);
    const float u = d * nzi.y;
    return __builtin_amdgcn_fmed3f(rintf(u), 0.0f, 3.0f);
}
// Sixteen codes -> one word with code k at bit 16*(k%2) + 2*(k/2): the two half-words are summed as exact
// binary32 numbers (code * 4^j < 2^16), one fused multiply-add per code, and converted once.
struct WordAcc {
    float lo = 0.f, hi = 0.f;
    __device__ inline void add(int k, float code)             // k: compile-time position 0..15
    {
        const float wgt = (float)(1 << (2 * (k >> 1)));
        if (k & 1) hi = __builtin_fmaf(code, wgt, hi); else lo = __builtin_fmaf(code, wgt, lo);
    }
    __device__ inline uint32_t word() const { return (uint32_t)lo | ((uint32_t)hi << 16); }
};

template <int G>
__global__ __launch_bounds__(256) void quantize_pack_kernel(QuantArgs a)
{
    constexpr int BT = G > 64 ? G : 64;               // tokens per workgroup
    constexpr int NCG = kD / G;                       // V channel groups per token
    constexpr int NPAR = (BT / G) * kD > BT * NCG ? (BT / G) * kD : BT * NCG;

    __shared__ __attribute__((aligned(16))) uint16_t tile[BT * kRow];
    __shared__ __attribute__((aligned(16))) float2 par[NPAR];      // (-zero, 1/scale) of every group

    const int u = blockIdx.y;
    const int tid = threadIdx.x;
    float one = 1.0f;
    asm volatile("" : "+v"(one));                       // (see quant_codef)
    int q0;
    const int n = tokens_to_append<G>(a, u, q0);
    const int i0 = blockIdx.x * BT;
    if (i0 >= n) return;
    const int nt = (n - i0 < BT) ? n - i0 : BT;        // multiple of G
    const int t0 = q0 + i0;                            // first destination token, multiple of G

    // ---------------- K: groups of G tokens per channel.  Statistics: one thread per (group, channel pair),
    // packed fp16 min / max (exact) down the G tokens.
    size_t off[BT / 16];
    row_offsets(off, a, u, i0, nt);
    load_rows(tile, a.K, off, nt);
    __syncthreads();
    for (int gi = tid; gi < (nt / G) * (kD / 2); gi += 256) {
        const int g = gi / (kD / 2), cp = gi % (kD / 2);
        const uint32_t *col = reinterpret_cast<const uint32_t *>(tile + g * G * kRow) + cp;
        qh2 mn = as_qh2(col[0]), mx = mn;
#pragma unroll 8
        for (int i = 1; i < G; i++) {
            const qh2 x = as_qh2(col[i * (kRow / 2)]);
            mn = pk_min(mn, x);
            mx = pk_max(mx, x);
        }
#pragma unroll
        for (int e = 0; e < 2; e++) {
            const int c = 2 * cp + e;
            uint16_t sh, zh; float inv, zf;
            group_params((float)mn[e], (float)mx[e], sh, zh, inv, zf);
            const size_t o = ((size_t)u * (a.Tcap / G) + (size_t)(t0 / G + g)) * kD + k_meta_pos(G, c);
            a.Ks[o] = sh;
            a.Kz[o] = zh;
            par[g * kD + c] = float2{-zf, inv};
        }
    }
    __syncthreads();
    // (the two word-building passes exist twice: for a full block of BT tokens, where every index split below is a
    // shift, and for the ragged last block of a unit, where they are divisions by run-time values)
    auto k_words = [&a, tid, u, t0, one](auto ntc) {
        // one thread per (token, word): the word's 16 channels are contiguous in the tile row and in par
        const int nt = ntc;
        uint32_t *Kc = a.Kc + (size_t)u * kc_words(a.Tcap);
        const int npair = nt / 2;
        for (int wi = tid; wi < nt * 8; wi += 256) {
            const int wq = wi & 3;
            const int pr = (wi >> 2) % npair;
            const int ch = wi / (4 * npair);           // 0..3 = 2*(token parity) + (word half)
            const int i = 2 * pr + (ch >> 1);
            const int w = (ch & 1) * 4 + wq;
            const uint4 *xs = reinterpret_cast<const uint4 *>(tile + i * kRow + 16 * w);
            const float4 *ps = reinterpret_cast<const float4 *>(par + (i / G) * kD + 16 * w);
            WordAcc acc;
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint4 x4 = xs[h];
                const uint32_t xw[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
                for (int k2 = 0; k2 < 4; k2++) {
                    const qh2 x = as_qh2(xw[k2]);
                    const float4 p = ps[4 * h + k2];   // (zero, inv) of channels 8h + 2k2, 8h + 2k2 + 1
                    acc.add(8 * h + 2 * k2, quant_codef(x[0], float2{p.x, p.y}, one));
                    acc.add(8 * h + 2 * k2 + 1, quant_codef(x[1], float2{p.z, p.w}, one));
                }
            }
            Kc[k_word_index(t0 + i, w)] = acc.word();
        }
    };
    if (nt == BT) k_words(std::integral_constant<int, BT>()); else k_words(nt);
    __syncthreads();

    // ---------------- V: groups of G channels per token.  Statistics: one thread per (token, channel group),
    // the G values read 8 at a time.
    load_rows(tile, a.V, off, nt);
    __syncthreads();
    for (int gi = tid; gi < nt * NCG; gi += 256) {
        const int i = gi / NCG, cg = gi % NCG;
        const uint4 *xs = reinterpret_cast<const uint4 *>(tile + i * kRow + cg * G);
        qh2 mn, mx;
#pragma unroll
        for (int k = 0; k < G / 8; k++) {
            const uint4 x4 = xs[k];
            const qh2 x0 = as_qh2(x4.x), x1 = as_qh2(x4.y), x2 = as_qh2(x4.z), x3 = as_qh2(x4.w);
            const qh2 lo = pk_min(pk_min(x0, x1), pk_min(x2, x3)), hi = pk_max(pk_max(x0, x1), pk_max(x2, x3));
            mn = k ? pk_min(mn, lo) : lo;
            mx = k ? pk_max(mx, hi) : hi;
        }
        const float mnf = fminf((float)mn[0], (float)mn[1]), mxf = fmaxf((float)mx[0], (float)mx[1]);
        uint16_t sh, zh; float inv, zf;
        group_params(mnf, mxf, sh, zh, inv, zf);
        const size_t o = ((size_t)u * a.Tcap + (size_t)(t0 + i)) * NCG + cg;
        a.Vs[o] = sh;
        a.Vz[o] = zh;
        par[gi] = float2{-zf, inv};
    }
    __syncthreads();
    auto v_words = [&a, tid, u, t0, one](auto ntc) {
        // one thread per (block of 16 tokens, channel pair): two words
        const int nt = ntc;
        uint32_t *Vc = a.Vc + (size_t)u * vc_words(a.Tcap);
        const int nb = nt / 16;
        for (int wi = tid; wi < nb * (kD / 2); wi += 256) {
            const int bl = wi % nb, cp = wi / nb;
            const int cg = (2 * cp) / G;
            const uint32_t *col = reinterpret_cast<const uint32_t *>(tile + 16 * bl * kRow) + cp;
            const float2 *ps = par + (16 * bl) * NCG + cg;
            WordAcc acc0, acc1;
#pragma unroll
            for (int p = 0; p < 16; p++) {
                const qh2 x = as_qh2(col[p * (kRow / 2)]);
                const float2 zi = ps[p * NCG];
                acc0.add(p, quant_codef(x[0], zi, one));
                acc1.add(p, quant_codef(x[1], zi, one));
            }
            Vc[v_word_index(t0 / 16 + bl, 2 * cp)] = acc0.word();
            Vc[v_word_index(t0 / 16 + bl, 2 * cp + 1)] = acc1.word();
        }
    };
    if (nt == BT) v_words(std::integral_constant<int, BT>()); else v_words(nt);
}

// Runs after every workgroup of quantize_pack_kernel has finished (next kernel on the stream).
template <int G>
__global__ void update_lengths_kernel(QuantArgs a, int units)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    int q0;
    const int n = tokens_to_append<G>(a, u, q0);
    if (n == 0) return;
    a.q_len[u] = q0 + n;
    if (a.flush) a.r_len[u] = 0;
}

// One workgroup of 64 threads per group of 2 units: thread = (unit, K or V, 16-byte piece).  The new rows
// are requested together with the length, so the kernel costs one memory round trip plus the store.
__global__ __launch_bounds__(64) void append_residual_kernel(const uint16_t *k_new, const uint16_t *v_new,
                                                             uint16_t *Rk, uint16_t *Rv, int32_t *r_len,
                                                             int Rcap, int units)
{
    const int tid = threadIdx.x;
    const int u = blockIdx.x * 2 + (tid >> 5);
    if (u >= units) return;
    const int which = (tid >> 4) & 1, piece = tid & 15;
    const uint4 row = reinterpret_cast<const uint4 *>((which ? v_new : k_new) + (size_t)u * kD)[piece];
    const int r = r_len[u];
    if (r < 0 || r >= Rcap) return;
    uint16_t *dst = (which ? Rv : Rk) + ((size_t)u * Rcap + r) * kD;
    reinterpret_cast<uint4 *>(dst)[piece] = row;
    // every thread of the unit has its r in a register by now (the loads above were waited for), so the
    // length can be bumped without a barrier
    if ((tid & 31) == 0) r_len[u] = r + 1;
}

template <int G>
static int launch_quantize_g(const QuantArgs &a, int units, int max_tok, hipStream_t st)
{
    constexpr int BT = G > 64 ? G : 64;
    dim3 grid((max_tok + BT - 1) / BT, units);
    hipLaunchKernelGGL(quantize_pack_kernel<G>, grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL(update_lengths_kernel<G>, dim3((units + 255) / 256), dim3(256), 0, st, a, units);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

int launch_quantize(const minikv_shape &s, const minikv_f16 *K, const minikv_f16 *V, int64_t L,
                    const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, int32_t max_tok,
                    const minikv_cache &c, bool flush, hipStream_t st)
{
    QuantArgs a;
    a.K = K; a.V = V; a.idx = idx; a.n_tok = n_tok;
    a.Kc = c.Kc; a.Vc = c.Vc; a.Ks = c.Ks; a.Kz = c.Kz; a.Vs = c.Vs; a.Vz = c.Vz;
    a.q_len = c.q_len; a.r_len = c.r_len;
    a.L = L; a.idx_stride = idx_stride; a.Tcap = s.Tcap; a.Rcap = s.Rcap; a.flush = flush ? 1 : 0;
    a.max_tok = max_tok;
    const int units = s.B * s.Hkv;
    switch (s.G) {
    case 16: return launch_quantize_g<16>(a, units, max_tok, st);
    case 32: return launch_quantize_g<32>(a, units, max_tok, st);
    case 64: return launch_quantize_g<64>(a, units, max_tok, st);
    case 128: return launch_quantize_g<128>(a, units, max_tok, st);
    }
    return MINIKV_EUNSUPPORTED;
}

int launch_append(const minikv_shape &s, const minikv_f16 *k_new, const minikv_f16 *v_new,
                  const minikv_cache &c, hipStream_t st)
{
    const int units = s.B * s.Hkv;
    hipLaunchKernelGGL(append_residual_kernel, dim3((units + 1) / 2), dim3(64), 0, st, k_new, v_new, c.Rk,
                       c.Rv, c.r_len, s.Rcap, units);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

}  // namespace minikv
