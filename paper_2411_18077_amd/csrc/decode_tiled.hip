// Decode attention over the packed 2-bit cache: the one-launch kernel of minikv_decode_attn (gfx950, wave64).
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
// Work split: a flat, weighted list of work items (passes of 128 quantized tokens, items of 64 fp16
// residual tokens) over all (batch, KV head) units is cut into equal ranges, one per single-wave
// workgroup; see "Work distribution" below.  Every wave keeps its own online-softmax state and the last
// wave to finish a unit merges the unit's partial results, all inside one launch.
//
// One pass of 128 quantized tokens, lane l of the wave:
//   K phase: the lane owns tokens 2l and 2l+1; four 128-bit loads bring their 2 x 8 code words.  Codes
//     are NOT converted: (word & (0x00030003 << 2j)) is used directly as two fp16 SUBNORMALS
//     code * 4^j * 2^-24 (j <= 4 keeps the field inside the mantissa; fields 5..7 come from the word
//     shifted right by 6), the 4^-j sits on the other operand and the 2^24 on the result.  The products
//     go to v_mfma_f32_4x4x4f16: 16 blocks = 64 tokens per instruction, lane = token, the 4 result
//     registers = 4 query heads, k = 4 channels.  The other operand, q_c * Ks[g,c] for (head, 4 channels),
//     is an exact fp16 pair (hi, lo) computed in registers by the lanes of the token's K group and handed
//     to the whole group by the instruction's block broadcast (cbsz / abid), so it never touches LDS;
//     the K scale / zero rows are stored so that each lane's channel quads are contiguous.
//   softmax: per-head wave maximum (DPP), lazy rescale of the accumulators, p = exp2(score - m).
//   V phase: the lane owns channels l and l+64.  ps[gc][h][t] = p * Vs * 2^4 * 4^-j(t) goes through LDS as
//     fp16 (written by the token lanes, read once by the lanes that supply it, again broadcast by the
//     instruction); the V words (16 tokens of one channel, even tokens in the low half-word) are masked
//     like the K words and multiplied 4 tokens x 4 heads at a time.  The zero-point term is accumulated
//     per lane in fp32 and reduced once per segment.
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
constexpr int kPsH = kPass + 4;        // halfs per (channel group, head) row of ps, padded
constexpr int kPsG = kNH * kPsH;       // halfs per channel group of ps (528: shifts 8 banks)
constexpr int kKRowH = kD + 8;         // halfs per staged residual key row (272 B: rows start 4 banks apart)

__device__ inline h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ inline uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// field j (0..7) of a half-word pair -> (shift inside the mantissa, use the >>6 copy?)
__host__ __device__ constexpr int fld_shift(int j) { return j <= 4 ? 2 * j : 2 * (j - 3); }
__host__ __device__ constexpr bool fld_shifted(int j) { return j > 4; }
// 4^-(shift/2): what the small operand is pre-multiplied by so that the masked subnormal needs no shift
__device__ inline float fld_scale(int j) { return 1.0f / (float)(1 << fld_shift(j)); }

__device__ inline h2 field(uint32_t w, uint32_t w6, int j)
{
    return as_h2((fld_shifted(j) ? w6 : w) & (0x00030003u << fld_shift(j)));
}

// ---- cross-lane reductions on the DPP data path (no LDS traffic)
template <int CTRL, int ROW_MASK = 0xF>
__device__ inline float dpp_mov(float old, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v),
                                                                  CTRL, ROW_MASK, 0xF, false));
}

// Four independent reductions at once, hand-scheduled: step k of all four values is issued back to back,
// so the two wait states a DPP read needs after a VALU write are always covered by the other three.
#define MINIKV_DPP4(op, ctrl)                                                     \
    "v_" op "_f32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %2, %2, %2 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %3, %3, %3 " ctrl " bank_mask:0xf\n"
#define MINIKV_ROW16(op)                                                          \
    MINIKV_DPP4(op, "quad_perm:[1,0,3,2] row_mask:0xf")                           \
    MINIKV_DPP4(op, "quad_perm:[2,3,0,1] row_mask:0xf")                           \
    MINIKV_DPP4(op, "row_half_mirror row_mask:0xf")                               \
    MINIKV_DPP4(op, "row_mirror row_mask:0xf")
#define MINIKV_WAVE64(op)                                                         \
    MINIKV_ROW16(op)                                                              \
    MINIKV_DPP4(op, "row_bcast:15 row_mask:0xa")                                  \
    MINIKV_DPP4(op, "row_bcast:31 row_mask:0xc")

__device__ inline float lane63(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// v[i] <- maximum of v[i] over the wave (wave-uniform)
__device__ inline void wave_max64x4(float v[4])
{
    asm volatile("s_nop 1\n" MINIKV_WAVE64("max") : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
    for (int i = 0; i < 4; i++) v[i] = lane63(v[i]);
}
// v[i] <- sum of v[i] over the wave (wave-uniform)
__device__ inline void wave_sum64x4(float v[4])
{
    asm volatile("s_nop 1\n" MINIKV_WAVE64("add") : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
    for (int i = 0; i < 4; i++) v[i] = lane63(v[i]);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; exp2(-inf) = 0

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

// The broadcast controls of the matrix instruction are immediates; these helpers turn the (unrolled,
// hence constant) block index into one.
#define MINIKV_MFMA_CASE(n) case n: acc = __builtin_amdgcn_mfma_f32_4x4x4f16(av, bv, acc, CB, n, 0); break;
template <int CB>
__device__ inline void mfma_bc(f4 &acc, h4 av, h4 bv, int abid)
{
    switch (abid) {
        MINIKV_MFMA_CASE(0) MINIKV_MFMA_CASE(1) MINIKV_MFMA_CASE(2) MINIKV_MFMA_CASE(3)
        MINIKV_MFMA_CASE(4) MINIKV_MFMA_CASE(5) MINIKV_MFMA_CASE(6) MINIKV_MFMA_CASE(7)
        MINIKV_MFMA_CASE(8) MINIKV_MFMA_CASE(9) MINIKV_MFMA_CASE(10) MINIKV_MFMA_CASE(11)
        MINIKV_MFMA_CASE(12) MINIKV_MFMA_CASE(13) MINIKV_MFMA_CASE(14) MINIKV_MFMA_CASE(15)
    }
}
template <int CB>
__device__ inline void mfma_k(f4 &acc0, f4 &acc1, h4 av, h4 b0, h4 b1, int abid)
{
    mfma_bc<CB>(acc0, av, b0, abid);
    mfma_bc<CB>(acc1, av, b1, abid);
}
template <int CB>
__device__ inline void mfma_v(f4 &o0, f4 &o1, h4 a0, h4 a1, h4 b0, h4 b1, int abid)
{
    mfma_bc<CB>(o0, a0, b0, abid);
    mfma_bc<CB>(o1, a1, b1, abid);
}

// ------------------------------------------------------------------------------------------------
constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

template <int N>
__device__ inline float dpp_ror_add(float v)              // v + (v rotated right by N lanes inside its row of 16)
{
    return v + dpp_mov<0x120 + N>(0.f, v);
}
template <int H>
__device__ inline float quad_bcast(float v)               // value of lane (4*(lane/4) + H)
{
    return dpp_mov<H * 0x55>(0.f, v);
}

// What one wave needs from global memory for the K half and the V half of one pass of 128 tokens.
template <int NKW>
struct KData {
    u4 kw[4];               // K code words of tokens 2*lane (kw[0..1]) and 2*lane+1 (kw[2..3])
    Words<NKW> ks, kz;      // this lane's bin of the K scale / zero row of its group
};
template <int NCG>
struct VData {
    u4 vw[2][2];            // V code words [channel lane / lane+64][64-token tile]: 4 blocks of 16 tokens each
    Words<NCG> vs, vz;      // V scale / zero of tokens 2*lane and 2*lane+1 (zero when past the end)
};

// ------------------------------------------------------------------------------------------------
// Work distribution ("flat list"): every unit (batch, KV head, set of 4 query heads) contributes
// ceil(T/128) quantized passes followed by ceil(R/64) residual items; the concatenation of all units'
// items is cut into gridDim.x equal ranges, one per single-wave workgroup.  A maximal run of items of one
// kind inside one unit and one wave is a "segment": it ends with one split-K partial (running max, sum,
// un-normalised output).  The segment that arrives last at its unit (device-scope ticket counter) merges
// the unit's partials and writes the fp16 output, so one kernel launch does the whole call and ragged
// lengths are balanced by construction.
struct UnitItems { int nq, nr; };
constexpr int kWQ = 2, kWR = 7;        // relative cost of a quantized pass (128 tokens, 12 KB) and a residual
                                       // item (64 fp16 tokens, 32 KB), measured

__device__ inline UnitItems unit_items(const DecArgs &a, int up)
{
    const int u = up >> a.hs_shift;
    const int T = clampi(a.q_len[u], 0, a.Tcap), R = clampi(a.r_len[u], 0, a.Rcap);
    return UnitItems{(T + kPass - 1) / kPass, (R + 63) / 64};
}
// P weight units are cut into NW = 2^nw_log ranges [w*P >> nw_log, (w+1)*P >> nw_log).
__device__ inline long range_start(int w, int P, int nw_log) { return ((long)w * P) >> nw_log; }
// wave that owns position i: binary32 estimate, then exact correction against the range bounds
__device__ inline int wave_of(long i, int P, int nw_log, float inv_p)
{
    int w = (int)((float)i * (float)(1 << nw_log) * inv_p);
    w = min(max(w, 0), (1 << nw_log) - 1);
    while (range_start(w, P, nw_log) > i) w--;
    while (range_start(w + 1, P, nw_log) <= i) w++;
    return w;
}

// wave-wide inclusive prefix sum of an int (lane 63 ends up with the total)
__device__ inline int wave_scan_i32(int v)
{
    asm volatile("s_nop 1\n"
                 "v_add_u32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n s_nop 1\n"
                 "v_add_u32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n s_nop 1\n"
                 "v_add_u32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n s_nop 1\n"
                 "v_add_u32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n s_nop 1\n"
                 "v_add_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n s_nop 1\n"
                 "v_add_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n"
                 : "+v"(v));
    return v;
}
__device__ inline int wave_sum_i32(int v) { return __builtin_amdgcn_readlane(wave_scan_i32(v), 63); }
// Split-K partials travel between workgroups (possibly on different XCDs, each with its own L2) inside
// one launch.  They are written and read with device-scope relaxed atomics, which the hardware performs
// at the device-coherent level instead of in the XCD-local L2, so no L2 write-back or invalidate is needed;
// the writer only has to wait for its stores to be acknowledged before it takes the ticket.
__device__ inline float ld_agent(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float2 ld_agent2(const float *p)      // two consecutive floats, p 8-byte aligned
{
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return float2{__builtin_bit_cast(float, (uint32_t)v), __builtin_bit_cast(float, (uint32_t)(v >> 32))};
}
__device__ inline void st_agent(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Split-K partial of (slot, head): [0] running max (base-2 domain), [1] sum of weights, [4..131] output.
__device__ inline float *slot_ptr(const DecArgs &a, int slot, int h)
{
    return a.ws + ((size_t)slot * kNH + h) * kPartialStride;
}

#ifdef MINIKV_TIMELINE
__device__ long long g_timeline[16384 * 8];
#define TL(slot) do { if (threadIdx.x == 0) g_timeline[(size_t)(blockIdx.x % 16384) * 8 + (slot)] = __builtin_readcyclecounter(); } while (0)
__device__ long long g_tl2[16384 * 16];
#define TL2(slot) do { if (threadIdx.x == 0) g_tl2[(size_t)(blockIdx.x % 16384) * 16 + (slot)] = __builtin_readcyclecounter(); } while (0)
#else
#define TL(slot) do {} while (0)
#define TL2(slot) do {} while (0)
#endif

template <int G, bool LO>
__global__ __launch_bounds__(64, 2) void decode_stream_kernel(DecArgs a)
{
    // K side: a K group spans G/2 token-lanes = BGK blocks of 4 lanes.  Block j of a group supplies the
    // A operand (4 heads x 4 channels of q*Ks) of k-steps j, j+BGK, ...; the matrix instruction
    // broadcasts it to the other blocks of the group (cbsz = log2 BGK, abid = j).
    constexpr int BGK = G / 8, CBK = ilog2(BGK), NKR = 32 / BGK;
    // V side: the lanes' channels lane, lane+64 share a channel group in runs of BGV blocks.
    constexpr int BGV = G / 4 < 16 ? G / 4 : 16, CBV = ilog2(BGV), NVR = 32 / BGV;
    constexpr int NCG = kD / G;
    constexpr int NKW = NKR * 2;                           // words of one lane's slice of a K meta row
    typedef KData<NKW> KD;
    typedef VData<NCG> VD;

    extern __shared__ __attribute__((aligned(16))) _Float16 lds[];
    _Float16 *ps = lds;                                    // [NCG][kNH][kPsH] halfs (quantized segments)

    const int lane = threadIdx.x, w = blockIdx.x;
    const int NU = a.units * a.hsets;
    TL(0);

    // ---------------- total weight of all items; units without any token get their zeros here
    auto unit_weight = [&](int uu) -> int {
        if (uu >= NU) return 0;
        const UnitItems it = unit_items(a, uu);
        return kWQ * it.nq + kWR * it.nr;
    };
    int mine = 0;
    for (int base = 0; base < NU; base += 256) {
        int n[4];
#pragma unroll
        for (int k = 0; k < 4; k++) n[k] = unit_weight(base + 64 * k + lane);
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int uu = base + 64 * k + lane;
            mine += n[k];
            if (uu < NU && n[k] == 0 && uu % (int)gridDim.x == w) {
                const int u = uu >> a.hs_shift, hs = uu & (a.hsets - 1);
                const int bi = (int)fast_div((uint32_t)u, a.hkv_magic, a.hkv_shift);
                const int bq0 = bi * a.Hq + (u - bi * a.Hkv) * a.rep + hs * kNH;
                const int nh = min(kNH, a.rep - hs * kNH);
                for (int i = 0; i < nh * kD; i++) a.out[(size_t)bq0 * kD + i] = 0;
            }
        }
    }
    const int P = wave_sum_i32(mine);
    // The weight line is cut into NW ranges, each at least one residual item long, so that every wave
    // between the first and the last wave of a unit's passes (or residual items) owns one of them.
    // NW is a power of two so that the cuts need no division.
    if (P == 0) return;
    const int nw_cap = max(1, min((int)gridDim.x, P / kWR));
    const int nw_log = 31 - __builtin_clz(nw_cap), NW = 1 << nw_log;
    if (w >= NW) return;
    const long start = range_start(w, P, nw_log), end = range_start(w + 1, P, nw_log);
    const float inv_p = 1.0f / (float)P;

    // ---------------- the unit whose weight span holds position `start`
    int up = -1;
    long ib = 0;                                           // position of the unit's first item
    {
        long running = 0;
        for (int base = 0; base < NU && up < 0; base += 64) {
            const int n = unit_weight(base + lane);
            const int incl = wave_scan_i32(n);
            const long excl = running + incl - n;
            const bool hit = n > 0 && start >= excl && start < excl + n;
            const unsigned long long mask = __ballot(hit);
            if (mask) {
                const int src = __ffsll((long long)mask) - 1;
                up = base + src;
                ib = running + __shfl(incl - n, src);
            }
            running += __builtin_amdgcn_readlane(incl, 63);
        }
    }
    TL(1);

    const int blk4 = lane >> 2, row = lane & 3;            // block of 4 lanes; row = query head this lane
                                                           // supplies as A operand
    const int gl = blk4 / BGK;                             // K group (of the pass) of this lane's tokens
    const int bbk = blk4 % BGK;                            // this lane's bin of k-steps: bbk, bbk+BGK, ...
    const int bbv = blk4 % BGV;                            // same on the V side (k-steps of 4 tokens)
    const int cg0 = lane / G;                              // channel groups of channels lane, lane+64
    const int cg1 = (lane + 64) / G;
    // Tokens 2*lane, 2*lane+1 are field j = lane & 7 of their V word.  The weights of this lane carry the
    // constant factor 2^lg = 16 * 4^-shift so that the masked V field needs no shift; the lane's running
    // sums l and oz carry the same factor and are unscaled once per segment.
    const float lg = 4.0f - (float)fld_shift(lane & 7);
    const float unlg = fast_exp2(-lg);
    const float kscale = a.c1 * 16777216.0f;               // undo the 2^-24 of the subnormal code fields
    const float vun = 16777216.0f / 16.0f;                 // 2^24 (subnormal fields) / 2^4 (ps headroom)

    // A wave owns the items whose start position lies in [start, end).
    for (; up < NU && ib < end; up++) {
        TL2(8);
        const UnitItems it = unit_items(a, up);
        const int wt = kWQ * it.nq + kWR * it.nr;
        if (wt == 0) continue;
        const long rb = ib + (long)kWQ * it.nq;            // position of the unit's first residual item
        // (the offsets are clamped to the unit's span first, so 32-bit arithmetic suffices)
        const int span = wt + kWR;
        const int ds = (int)min((long)span, max(0L, start - ib)), de = (int)min((long)span, max(0L, end - ib));
        const int j0 = min(it.nq, (ds + kWQ - 1) / kWQ), j1 = min(it.nq, (de + kWQ - 1) / kWQ);
        const int dq = kWQ * it.nq;
        const int r0 = min(it.nr, (max(0, ds - dq) + kWR - 1) / kWR), r1 = min(it.nr, (max(0, de - dq) + kWR - 1) / kWR);
        const int u = up >> a.hs_shift, hs = up & (a.hsets - 1);
        const int bi = (int)fast_div((uint32_t)u, a.hkv_magic, a.hkv_shift);
        const int bq0 = bi * a.Hq + (u - bi * a.Hkv) * a.rep + hs * kNH;
        const int nheads = min(kNH, a.rep - hs * kNH);
        // segments of this unit: waves first..last of its quantized items and of its residual items
        const int wq0 = it.nq ? wave_of(ib, P, nw_log, inv_p) : 0, wq1 = it.nq ? wave_of(rb - kWQ, P, nw_log, inv_p) : -1;
        const int wr0 = it.nr ? wave_of(rb, P, nw_log, inv_p) : 0, wr1 = it.nr ? wave_of(ib + wt - kWR, P, nw_log, inv_p) : -1;
        const int expected = (wq1 - wq0 + 1) + (wr1 - wr0 + 1);
        const long ib_next = ib + wt;

      TL2(9);
      for (int kind = 0; kind < 2; kind++) {
        if (kind == 0 ? j0 >= j1 : r0 >= r1) continue;

        float m[kNH], lsum[kNH];                           // result of the segment (wave-uniform m, lsum)
        float oa[kNH], ob[kNH];                            // un-normalised output of two channels per lane
        int ca, cb;                                        // which two channels

        if (kind == 0) {
            // =============================== quantized passes j0 .. j1-1 of unit u
            const int j = j0;
            const int T = clampi(a.q_len[u], 0, a.Tcap);
            const int t_end = T;
            const uint32_t *Kc = a.Kc + (size_t)u * kc_words(a.Tcap);
            const uint32_t *Vc = a.Vc + (size_t)u * vc_words(a.Tcap);
            const uint16_t *Ks = a.Ks + (size_t)u * (a.Tcap / G) * kD;
            const uint16_t *Kz = a.Kz + (size_t)u * (a.Tcap / G) * kD;
            const uint16_t *Vs = a.Vs + (size_t)u * a.Tcap * NCG;
            const uint16_t *Vz = a.Vz + (size_t)u * a.Tcap * NCG;

            // this lane's query values: head `row`, the channels of its k-steps, raw and pre-scaled by the
            // 4^-j of the code field (channel pair (c, c+1), c even, is field (c % 16) / 2 of its K word)
            h2 qraw[NKR][2], qscl[NKR][2];
#pragma unroll
            for (int i = 0; i < NKR; i++)
#pragma unroll
                for (int ep = 0; ep < 2; ep++) {
                    const int c = 4 * (bbk + BGK * i) + 2 * ep;
                    uint32_t bits = 0;
                    if (row < nheads) bits = *reinterpret_cast<const uint32_t *>(a.q + (size_t)(bq0 + row) * kD + c);
                    qraw[i][ep] = as_h2(bits);
                    qscl[i][ep] = qraw[i][ep] * (_Float16)fld_scale((c & 15) >> 1);
                }

            TL2(10);
            float l_lane[kNH];
            f4 O0 = {0.f, 0.f, 0.f, 0.f}, O1 = {0.f, 0.f, 0.f, 0.f};   // channel lane / lane+64, 4 heads each
            float oz[kNH][NCG];
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                m[h] = -1e30f; l_lane[h] = 0.f;
#pragma unroll
                for (int g = 0; g < NCG; g++) oz[h][g] = 0.f;
            }

            auto load_k = [&](int tp) -> KD {
                KD d;
                const u4 *ktile = reinterpret_cast<const u4 *>(Kc + (size_t)(tp >> 7) * 1024);
#pragma unroll
                for (int i = 0; i < 4; i++) d.kw[i] = ktile[i * 64 + lane];
                const bool gvalid = tp + gl * G < t_end;
                const size_t go = ((size_t)(tp / G) + (gvalid ? gl : 0)) * kD + bbk * (NKR * 4);
                d.ks = load_words<NKW>(Ks + go);
                d.kz = load_words<NKW>(Kz + go);
                return d;
            };
            auto load_v = [&](int tp) -> VD {
                VD d;
                const u4 *vtile = reinterpret_cast<const u4 *>(Vc + (size_t)(tp >> 6) * (4 * kD));
#pragma unroll
                for (int tl = 0; tl < 2; tl++) {
                    d.vw[0][tl] = vtile[tl * kD + lane];
                    d.vw[1][tl] = vtile[tl * kD + lane + 64];
                }
                // past the end the (clamped) load still happens and the value is masked to zero afterwards,
                // so that the number of loads in flight is the same on every path
                const bool valid = tp + 2 * lane < t_end;
                const size_t vo = (size_t)(valid ? tp + 2 * lane : tp) * NCG;
                d.vs = load_words<NCG>(Vs + vo);
                d.vz = load_words<NCG>(Vz + vo);
                return d;
            };

            float s0[kNH], s1[kNH];                        // scores of the lane's two tokens

            // ---------------- K phase: scores of tokens 2*lane, 2*lane+1 for the 4 heads
            auto k_phase = [&](const KD &d, int tp) {
                const bool valid = tp + 2 * lane < t_end;  // both tokens of the lane (t_end % 16 == 0)
                // A operands of this lane's k-steps (exact hi + lo split of q * Ks), qz = sum_c q_c Kz[g,c]
                h4 a_hi[NKR], a_lo[NKR];
                float qz = 0.f;
#pragma unroll
                for (int i = 0; i < NKR; i++) {
                    h2 hi[2], lo[2];
#pragma unroll
                    for (int ep = 0; ep < 2; ep++) {
                        const h2 ks2 = as_h2(d.ks.v[2 * i + ep]), kz2 = as_h2(d.kz.v[2 * i + ep]);
                        hi[ep] = qscl[i][ep] * ks2;
                        if constexpr (LO) lo[ep] = __builtin_elementwise_fma(qscl[i][ep], ks2, -hi[ep]);
                        qz = __builtin_amdgcn_fdot2(qraw[i][ep], kz2, qz, false);
                    }
                    a_hi[i] = h4{hi[0][0], hi[0][1], hi[1][0], hi[1][1]};
                    if constexpr (LO) a_lo[i] = h4{lo[0][0], lo[0][1], lo[1][0], lo[1][1]};
                }
                // sum the partial qz of the BGK blocks of the group (same row, lanes 4 apart)
                if constexpr (BGK == 2) qz += __shfl_xor(qz, 4);
                if constexpr (BGK >= 4) { qz = dpp_ror_add<4>(qz); qz = dpp_ror_add<8>(qz); }
                if constexpr (BGK >= 8) qz += __shfl_xor(qz, 16);
                if constexpr (BGK >= 16) qz += __shfl_xor(qz, 32);

                f4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int wd = 0; wd < 8; wd++) {
                    const uint32_t w0 = d.kw[wd >> 2][wd & 3], w1 = d.kw[2 + (wd >> 2)][wd & 3];
                    const uint32_t w0s = w0 >> 6, w1s = w1 >> 6;
#pragma unroll
                    for (int sq = 0; sq < 4; sq++) {
                        const int s = 4 * wd + sq;         // k-step: channels 4s..4s+3
                        const h2 x00 = field(w0, w0s, 2 * sq), x01 = field(w0, w0s, 2 * sq + 1);
                        const h2 x10 = field(w1, w1s, 2 * sq), x11 = field(w1, w1s, 2 * sq + 1);
                        const h4 b0 = {x00[0], x00[1], x01[0], x01[1]};
                        const h4 b1 = {x10[0], x10[1], x11[0], x11[1]};
                        mfma_k<CBK>(acc0, acc1, a_hi[s / BGK], b0, b1, s % BGK);
                        if constexpr (LO) mfma_k<CBK>(acc0, acc1, a_lo[s / BGK], b0, b1, s % BGK);
                    }
                }
                const float zz[kNH] = {quad_bcast<0>(qz) * a.c1, quad_bcast<1>(qz) * a.c1,
                                       quad_bcast<2>(qz) * a.c1, quad_bcast<3>(qz) * a.c1};
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    s0[h] = valid ? acc0[h] * kscale + zz[h] : -INFINITY;
                    s1[h] = valid ? acc1[h] * kscale + zz[h] : -INFINITY;
                }
            };

            // ---------------- softmax update, ps table, V products
            auto v_phase = [&](const VD &d, int tp) {
                const bool valid = tp + 2 * lane < t_end;
                float mn[kNH];
                bool grow = false;
#pragma unroll
                for (int h = 0; h < kNH; h++) mn[h] = fmaxf(s0[h], s1[h]);
                wave_max64x4(mn);
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    mn[h] = fmaxf(m[h], mn[h]);
                    grow |= mn[h] > m[h];
                }
                if (grow) {                                // wave-uniform
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float sc = fast_exp2(m[h] - mn[h]);
                        l_lane[h] *= sc;
                        O0[h] *= sc;
                        O1[h] *= sc;
#pragma unroll
                        for (int g = 0; g < NCG; g++) oz[h][g] *= sc;
                        m[h] = mn[h];
                    }
                }
                {
                    // (vs, vz) words hold [token 2l: NCG halfs][token 2l+1: NCG halfs]; pair them per group
                    h2 vsp[NCG], vzp[NCG];
#pragma unroll
                    for (int g = 0; g < NCG; g++) {
                        const int i0 = g, i1 = NCG + g;    // half index of (token 0, g) and (token 1, g)
                        const uint32_t sel = ((i0 & 1) ? 0x00000302u : 0x00000100u) | ((i1 & 1) ? 0x07060000u : 0x05040000u);
                        const uint32_t sv = __builtin_amdgcn_perm(d.vs.v[i1 >> 1], d.vs.v[i0 >> 1], sel);
                        const uint32_t zv = __builtin_amdgcn_perm(d.vz.v[i1 >> 1], d.vz.v[i0 >> 1], sel);
                        vsp[g] = as_h2(valid ? sv : 0u);
                        vzp[g] = as_h2(valid ? zv : 0u);
                    }
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float mo = m[h] - lg;
                        const float p0 = fast_exp2(s0[h] - mo), p1 = fast_exp2(s1[h] - mo);   // masked: 0
                        l_lane[h] += p0 + p1;
                        const h2 ph = {(_Float16)p0, (_Float16)p1};
#pragma unroll
                        for (int g = 0; g < NCG; g++) {
                            *reinterpret_cast<h2 *>(ps + g * kPsG + h * kPsH + 2 * lane) = ph * vsp[g];
                            oz[h][g] = __builtin_amdgcn_fdot2(ph, vzp[g], oz[h][g], false);
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();

                // A operands of this lane's V k-steps (4 tokens each): ps[channel group][head row][tokens]
                h4 a0[NVR], a1[NVR];
#pragma unroll
                for (int i = 0; i < NVR; i++) {
                    const int tok = 4 * (bbv + BGV * i);
                    a0[i] = *reinterpret_cast<const h4 *>(ps + cg0 * kPsG + row * kPsH + tok);
                    a1[i] = *reinterpret_cast<const h4 *>(ps + cg1 * kPsG + row * kPsH + tok);
                }
#pragma unroll
                for (int blk = 0; blk < 8; blk++) {
                    const uint32_t v0 = d.vw[0][blk >> 2][blk & 3], v1 = d.vw[1][blk >> 2][blk & 3];
                    const uint32_t v0s = v0 >> 6, v1s = v1 >> 6;
#pragma unroll
                    for (int kq = 0; kq < 4; kq++) {
                        const int ks = 4 * blk + kq;       // k-step: tokens 4ks..4ks+3 of the pass
                        const h2 x00 = field(v0, v0s, 2 * kq), x01 = field(v0, v0s, 2 * kq + 1);
                        const h2 x10 = field(v1, v1s, 2 * kq), x11 = field(v1, v1s, 2 * kq + 1);
                        const h4 b0 = {x00[0], x00[1], x01[0], x01[1]};
                        const h4 b1 = {x10[0], x10[1], x11[0], x11[1]};
                        mfma_v<CBV>(O0, O1, a0[ks / BGV], a1[ks / BGV], b0, b1, ks % BGV);
                    }
                }
                __builtin_amdgcn_wave_barrier();
            };

            // Loads run one phase ahead of their use and are issued on every path (the last iteration
            // re-requests its own tile), so the number in flight is always the same.
            {
                auto tp_of = [&](int jj) { return (jj < j1 ? jj : j1 - 1) * kPass; };
                KD kd = load_k(tp_of(j));
                VD vd = load_v(tp_of(j));
                TL(2);
                for (int jj = j; jj < j1; jj++) {
                    const int tp = jj * kPass;
                    if (jj == j) TL2(11);
                    k_phase(kd, tp);
                    if (jj == j) TL2(12);
                    kd = load_k(tp_of(jj + 1));
                    v_phase(vd, tp);
                    vd = load_v(tp_of(jj + 1));
                }
            }

            TL(3);
            // finish the segment: undo operand scalings, add the zero-point term
#pragma unroll
            for (int h = 0; h < kNH; h++) lsum[h] = l_lane[h] * unlg;
            wave_sum64x4(lsum);
#pragma unroll
            for (int g = 0; g < NCG; g++) {
                float zs[kNH];
#pragma unroll
                for (int h = 0; h < kNH; h++) zs[h] = oz[h][g] * unlg;
                wave_sum64x4(zs);
#pragma unroll
                for (int h = 0; h < kNH; h++) oz[h][g] = zs[h];    // now the wave total (uniform)
            }
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                float z0 = 0.f, z1 = 0.f;
#pragma unroll
                for (int g = 0; g < NCG; g++) {
                    z0 = (g == cg0) ? oz[h][g] : z0;
                    z1 = (g == cg1) ? oz[h][g] : z1;
                }
                oa[h] = O0[h] * vun + z0;
                ob[h] = O1[h] * vun + z1;
            }
            ca = lane; cb = lane + 64;
        } else {
            // =============================== residual items (64 fp16 tokens each) of unit u:
            // Algorithm 1's R_K t_Q^T and A_unquant R_V on the vector ALU.  This path runs rarely, so it
            // is written as compact loops (small code) around fully coalesced loads: the 64 key rows, then
            // the 64 value rows, are fetched 4 rows per instruction (16 lanes x 16 B per row) and staged in
            // LDS; lane = token for the scores, lane = channel pair for the values.
            const int R = clampi(a.r_len[u], 0, a.Rcap);
            _Float16 *qh = lds;                            // [kNH][128] halfs
            _Float16 *rows = lds + kNH * kD;               // [64][kKRowH] halfs: key rows, then value rows
            for (int i = lane; i < kNH * kD; i += 64) {
                const int h = i / kD;
                qh[i] = (h < nheads) ? __builtin_bit_cast(_Float16, a.q[(size_t)(bq0 + h) * kD + i % kD]) : (_Float16)0.f;
            }
            __builtin_amdgcn_wave_barrier();
            const uint16_t *Rk = a.Rk + (size_t)u * a.Rcap * kD;
            const uint16_t *Rv = a.Rv + (size_t)u * a.Rcap * kD;
#pragma unroll
            for (int h = 0; h < kNH; h++) { m[h] = -1e30f; lsum[h] = 0.f; oa[h] = 0.f; ob[h] = 0.f; }
            TL(2);
            const int rsub = lane >> 4, piece = lane & 15;  // row within a group of 4, 16-byte piece of the row

#pragma unroll 1
            for (int ri = r0; ri < r1; ri++) {
                const int t0 = ri * 64;
                const bool valid = t0 + lane < R;
                if (ri == r0) TL2(0);
                Words<64> g;
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int rr = t0 + 4 * i + rsub;
                    const uint4 x = reinterpret_cast<const uint4 *>(Rk + (size_t)(rr < R ? rr : 0) * kD)[piece];
                    g.v[4 * i] = x.x; g.v[4 * i + 1] = x.y; g.v[4 * i + 2] = x.z; g.v[4 * i + 3] = x.w;
                }
#pragma unroll
                for (int i = 0; i < 16; i++)
                    *reinterpret_cast<uint4 *>(rows + (4 * i + rsub) * kKRowH + piece * 8) =
                        uint4{g.v[4 * i], g.v[4 * i + 1], g.v[4 * i + 2], g.v[4 * i + 3]};
                // the value rows are requested now and travel while the scores are computed
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int rr = t0 + 4 * i + rsub;
                    const uint4 x = reinterpret_cast<const uint4 *>(Rv + (size_t)(rr < R ? rr : 0) * kD)[piece];
                    g.v[4 * i] = x.x; g.v[4 * i + 1] = x.y; g.v[4 * i + 2] = x.z; g.v[4 * i + 3] = x.w;
                }
                __builtin_amdgcn_wave_barrier();
                if (ri == r0) TL2(1);

                float acc[kNH] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
                for (int i = 0; i < 16; i++) {
                    const u4 kk = *reinterpret_cast<const u4 *>(rows + lane * kKRowH + i * 8);
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const u4 qq = *reinterpret_cast<const u4 *>(qh + h * kD + i * 8);
#pragma unroll
                        for (int p = 0; p < 4; p++)
                            acc[h] = __builtin_amdgcn_fdot2(as_h2(qq[p]), as_h2(kk[p]), acc[h], false);
                    }
                }
                __builtin_amdgcn_wave_barrier();
                if (ri == r0) TL2(2);
#pragma unroll
                for (int i = 0; i < 16; i++)
                    *reinterpret_cast<uint4 *>(rows + (4 * i + rsub) * kKRowH + piece * 8) =
                        uint4{g.v[4 * i], g.v[4 * i + 1], g.v[4 * i + 2], g.v[4 * i + 3]};
                if (ri == r0) TL2(3);

                float mn[kNH];
                bool grow = false;
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    acc[h] = valid ? acc[h] * a.c1 : -INFINITY;
                    mn[h] = acc[h];
                }
                wave_max64x4(mn);
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    mn[h] = fmaxf(m[h], mn[h]);
                    grow |= mn[h] > m[h];
                }
                if (grow) {
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float sc = fast_exp2(m[h] - mn[h]);
                        lsum[h] *= sc; oa[h] *= sc; ob[h] *= sc;
                        m[h] = mn[h];
                    }
                }
                float pr[kNH];                             // weight of this lane's token (0 past the end)
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    pr[h] = fast_exp2(acc[h] - m[h]);
                    lsum[h] += pr[h];
                }
                __builtin_amdgcn_wave_barrier();
                if (ri == r0) TL2(4);
                // values: the weight of token tt is read from lane tt (wave-uniform operand)
#pragma unroll 16
                for (int tt = 0; tt < 64; tt++) {
                    const h2 v = as_h2(*reinterpret_cast<const uint32_t *>(rows + tt * kKRowH + 2 * lane));
                    const float v0 = (float)v[0], v1 = (float)v[1];
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float ph = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pr[h]), tt));
                        oa[h] += ph * v0;
                        ob[h] += ph * v1;
                    }
                }
                __builtin_amdgcn_wave_barrier();
                if (ri == r0) TL2(5);
            }
            TL(3);
            wave_sum64x4(lsum);
            ca = 2 * lane; cb = 2 * lane + 1;
        }

        TL(4);
#ifdef MINIKV_TIMELINE
        if (lane == 0) g_timeline[(size_t)(blockIdx.x % 16384) * 8 + 7] = kind * 1000 + expected;
#endif
        // =============================== publish the segment
        if (expected == 1) {
            // the only segment of its unit: normalise and write the result directly
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                if (h < nheads) {
                    const float inv = lsum[h] > 0.f ? 1.0f / lsum[h] : 0.f;
                    a.out[(size_t)(bq0 + h) * kD + ca] = __half_as_ushort(__float2half_rn(oa[h] * inv));
                    a.out[(size_t)(bq0 + h) * kD + cb] = __half_as_ushort(__float2half_rn(ob[h] * inv));
                }
            }
        } else {
            const int slot = w + 2 * up + kind;
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                if (h < nheads) {
                    float *pp = slot_ptr(a, slot, h);
                    st_agent(pp + 4 + ca, oa[h]);
                    st_agent(pp + 4 + cb, ob[h]);
                    if (lane == 0) { st_agent(pp, m[h]); st_agent(pp + 1, lsum[h]); }
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // all stores acknowledged ...
            int old = 0;
            if (lane == 0) old = atomicAdd(a.cnt + up, 1);           // ... before the ticket is taken
            old = __shfl(old, 0);
            if (old == expected - 1) {
                // last segment of the unit to arrive: merge all partials, write the output.  Lane s fetches
                // (max, sum) of segment s, which gives every segment's weight; the output vectors (channels
                // 2*lane, 2*lane+1 per lane) of up to 16 segments are requested in the same round trip.
                const int nsq = wq1 - wq0 + 1;
                auto slot_of = [&](int sg) { return sg < nsq ? wq0 + sg + 2 * up : wr0 + (sg - nsq) + 2 * up + 1; };
                float M[kNH], L[kNH], Oa[kNH], Ob[kNH];
#pragma unroll
                for (int h = 0; h < kNH; h++) { M[h] = -1e30f; L[h] = 0.f; Oa[h] = 0.f; Ob[h] = 0.f; }
                constexpr int MB = 16;
#pragma unroll 1
                for (int base = 0; base < expected; base += MB) {
                    const int cnt = min(MB, expected - base);
                    const int sg = base + lane;
                    const bool has = lane < cnt;
                    const int my_slot = slot_of(has ? sg : base);
                    float ms[kNH], ls[kNH], cm[kNH];
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float2 ml = ld_agent2(slot_ptr(a, my_slot, h < nheads ? h : 0));
                        const bool on = has && h < nheads;
                        ms[h] = on ? ml.x : -1e30f;
                        ls[h] = on ? ml.y : 0.f;
                    }
                    float2 x[MB][kNH];
#pragma unroll
                    for (int k = 0; k < MB; k++) {
                        const int sl = slot_of(base + (k < cnt ? k : 0));      // clamped; weight zeroed below
#pragma unroll
                        for (int h = 0; h < kNH; h++) x[k][h] = ld_agent2(slot_ptr(a, sl, h < nheads ? h : 0) + 4 + 2 * lane);
                    }
#pragma unroll
                    for (int h = 0; h < kNH; h++) cm[h] = ms[h];
                    wave_max64x4(cm);
                    float wgt[kNH], lw[kNH];
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float Mn = fmaxf(M[h], cm[h]);
                        const float so = fast_exp2(M[h] - Mn);
                        wgt[h] = fast_exp2(ms[h] - Mn);
                        lw[h] = ls[h] * wgt[h];
                        L[h] *= so; Oa[h] *= so; Ob[h] *= so;
                        M[h] = Mn;
                    }
                    wave_sum64x4(lw);
#pragma unroll
                    for (int h = 0; h < kNH; h++) L[h] += lw[h];
#pragma unroll
                    for (int k = 0; k < MB; k++)
#pragma unroll
                        for (int h = 0; h < kNH; h++) {
                            const float wl = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wgt[h]), k));
                            const float wv = (k < cnt && h < nheads) ? wl : 0.f;
                            Oa[h] += x[k][h].x * wv;
                            Ob[h] += x[k][h].y * wv;
                        }
                }
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    if (h >= nheads) continue;
                    const float inv = L[h] > 0.f ? 1.0f / L[h] : 0.f;
                    const h2 r = {(_Float16)(Oa[h] * inv), (_Float16)(Ob[h] * inv)};
                    *reinterpret_cast<uint32_t *>(a.out + (size_t)(bq0 + h) * kD + 2 * lane) = as_u32(r);
                }
                if (lane == 0) a.cnt[up] = 0;              // ready for the next call
            }
        }
      }   // kind
        ib = ib_next;
    }
    TL(5);
}

#ifdef MINIKV_TIMELINE
extern "C" int minikv_debug_timeline(long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_timeline), (size_t)n * 8, 0, hipMemcpyDeviceToHost);
}
extern "C" int minikv_debug_timeline2(long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_tl2), (size_t)n * 8, 0, hipMemcpyDeviceToHost);
}
#endif

template <int G, bool LO>
static int launch_stream(DecArgs a, hipStream_t st)
{
    constexpr int NCG = kD / G;
    constexpr size_t q_bytes = (size_t)NCG * kPsG * 2;
    constexpr size_t r_bytes = (size_t)kNH * kD * 2 + (size_t)64 * kKRowH * 2;
    constexpr size_t lds_bytes = q_bytes > r_bytes ? q_bytes : r_bytes;
    auto kern = decode_stream_kernel<G, LO>;
    static int resident = 0;                               // single-wave workgroups the device holds at once
    if (resident == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 64, lds_bytes) != hipSuccess ||
            cus <= 0 || per_cu <= 0)
            return MINIKV_ELAUNCH;
        resident = cus * per_cu;
    }
    const long cap_items = (long)a.units * a.hsets * ((a.Tcap + kPass - 1) / kPass + (a.Rcap + 63) / 64);
    long nw = resident < kMaxStreamWaves ? resident : kMaxStreamWaves;
    if (nw > cap_items) nw = cap_items;
    if (nw < 1) nw = 1;
    hipLaunchKernelGGL(kern, dim3((unsigned)nw), dim3(64), lds_bytes, st, a);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

template <bool LO>
static int launch_stream_g(const DecArgs &a, int G, hipStream_t st)
{
    switch (G) {
    case 16: return launch_stream<16, LO>(a, st);
    case 32: return launch_stream<32, LO>(a, st);
    case 64: return launch_stream<64, LO>(a, st);
    case 128: return launch_stream<128, LO>(a, st);
    }
    return MINIKV_EUNSUPPORTED;
}

int launch_decode_tiled(const DecArgs &a, int G, int units, int variant, hipStream_t st)
{
    (void)units;
    switch (variant) {
    case 3: return launch_stream_g<true>(a, G, st);
    case 4: return launch_stream_g<false>(a, G, st);
    }
    return MINIKV_EINVAL;
}

}  // namespace minikv
