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
// Work split: single-wave workgroups, as many as the chip holds.  A flat, weighted list of work items
// (items of 64 fp16 residual tokens, passes of 128 quantized tokens) over all (batch, KV head) units is cut
// into equal ranges, one per wave; see "Work distribution" below.  Every wave keeps one online-softmax
// state per unit it touches and the last wave to finish a unit merges the unit's partial results, all
// inside one launch.
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
//     per lane in fp32 and reduced once per unit and wave.
//
// Input domain: every finite fp16 input.  The fp16 operands of the matrix instructions hold |q * Ks| < 65504
// and V scales < 4096 with the default scalings; a wave whose sums show an overflow repeats its share of the
// unit with range-normalised operands (see "Operand ranges" in the kernel).
#include <atomic>

#include "decode_wave.h"

namespace minikv {

// ------------------------------------------------------------------------------------------------
// Work distribution.  Every unit (batch, KV head, set of 4 query heads) has ceil(R/64) residual items and
// ceil(T/128) quantized passes; its span of the weight line holds the even residual items, the passes,
// then the odd residual items (so that the usual two items fall to two different waves).  The units'
// spans (kWR per residual item, kWQ per pass) are laid end to end and the line is cut into NW equal
// ranges, one per wave; a wave owns the items that START inside its range, so ragged lengths are balanced
// by construction.  What a wave does for one unit
// ends in one split-K partial (running max, sum, un-normalised output); the partial that arrives last at
// its unit (device-scope ticket counter) merges the unit's partials and writes the fp16 output, so one
// kernel launch does the whole call.  (Drawing passes from a per-unit counter instead was tried: a vector
// atomic per pass, even one whose result is needed a full pass later, slowed the pass loop by 40 %.)
struct UnitItems { int nq, nr, T, R, rn; };   // rn: residual row the fused step appends (-1: none)
constexpr int kSkew16 = 10;             // share (in sixteenths) of a wave pair's range given to its first wave
constexpr int kPassWeight = 2, kResidualWeight = 7;   // relative cost of a quantized pass (128 tokens, 12 KB) and a residual
                                       // item (64 fp16 tokens, 32 KB), measured

// Residual tokens a unit attends to: its stored ones, plus -- in the fused step -- the token this launch appends
// (when the buffer has room for it, as kv_append_residual would).
// A 32-bit word that no kernel of this launch writes, read through the constant address space: a wave-uniform
// address then gets a scalar load, which does not queue behind the wave's outstanding vector loads.  (Without
// this the fused step's stores of 32-bit words make the compiler read the lengths with vector loads.)
__device__ inline int load_const_i32(const int32_t *p)
{
    typedef const __attribute__((address_space(4))) int32_t *const_ptr;
    return *(const_ptr)(uintptr_t)p;
}
// (bit kAppBit of the result says that a token is appended, so that one register carries both facts)
constexpr int kAppBit = 20;
__device__ inline int res_len(bool APPEND, const DecArgs &a, int r)
{
    const int rc = clampi(r, 0, a.Rcap);
    return APPEND && r >= 0 && r < a.Rcap ? (rc + 1) | (1 << kAppBit) : rc;
}
__device__ inline UnitItems make_items(bool APPEND, int T, int Rtag)
{
    const int R = APPEND ? Rtag & ((1 << kAppBit) - 1) : Rtag;
    return UnitItems{(T + kPass - 1) / kPass, (R + 63) / 64, T, R, APPEND && (Rtag >> kAppBit) ? R - 1 : -1};
}
__device__ inline UnitItems unit_items(bool APPEND, const DecArgs &a, int up)
{
    const int u = up >> a.hs_shift;
    return make_items(APPEND, clampi(load_const_i32(a.q_len + u), 0, a.Tcap), res_len(APPEND, a, load_const_i32(a.r_len + u)));
}
// P weight units are cut into NW = 2^nw_log ranges.  Waves 2p and 2p+1 share the pair range
// [p*2P >> nw_log, (p+1)*2P >> nw_log); the first of them takes skew16/16 of it (8 = equal halves).
__device__ inline long range_start(int w, int P, int nw_log, int skew16)
{
    if (nw_log == 0) return w ? P : 0;
    const long s0 = ((long)(w >> 1) * P) >> (nw_log - 1);
    if (!(w & 1)) return s0;
    const long s1 = ((long)((w >> 1) + 1) * P) >> (nw_log - 1);
    return s0 + (((s1 - s0) * skew16) >> 4);
}
// wave that owns position i: binary32 estimate, then exact correction against the range bounds
__device__ inline int wave_of(long i, int P, int nw_log, float inv_p, int skew16)
{
    int w = (int)((float)i * inv_p);                       // inv_p = NW / P
    w = min(max(w, 0), (1 << nw_log) - 1);
    while (range_start(w, P, nw_log, skew16) > i) w--;
    while (range_start(w + 1, P, nw_log, skew16) <= i) w++;
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
// Split-K partial of (slot, head): [0] running max (base-2 domain), [1] sum of weights, [4..131] output.
__device__ inline float *slot_ptr(const DecArgs &a, int slot, int h)
{
    return a.ws + ((size_t)slot * kNH + h) * kPartialStride;
}

// Two waves per SIMD, except for G = 16, whose per-lane share of the K scale / zero rows and of q*Ks does not
// fit 256 registers: one wave per SIMD with the full register file runs 1.6x faster there than two that
// spill (the pass loop is bound by instruction issue, which one wave nearly saturates).
//
// PAIRED (units with at most two query heads, i.e. multi-head attention): the four rows of the K-phase
// A operand are (head 0 hi, head 0 lo, head 1 hi, head 1 lo) instead of four heads, so one matrix
// instruction does the work of the hi and the lo one, and the two result rows of a head are added afterwards.
//
// FUSED: the instance that serves the fused decode step (the plain call compiles none of it).  Inside it the
// step's code still hangs on the run-time flag a.append and not on the template parameter: measured on the
// 16 x 32768 workload, the instance built with the flag as a constant ran 3 us (7 %) slower, with or without a
// token to append -- the compiler then arranges the unit set-up and the residual item differently.
//
// FLAT: every item weighs 1.  A range of the work line must be at least one residual item long, so with the
// measured weights a small workload is cut into few ranges -- one sequence of 1024 tokens and 8 heads gets 16
// waves of 4 to 6 items each, 16 us of which 7 are items worked off one after the other.  When the whole
// launch cannot hold more items than half the waves the device holds, balance does not matter and
// parallelism does: with unit weights every item gets a wave of its own.
template <int G, bool LO, bool PAIRED, bool FUSED, bool FLAT>
__global__ __launch_bounds__(64, G == 16 ? 1 : 2) void decode_stream_kernel(DecArgs a)
{
    constexpr int kWQ = FLAT ? 1 : kPassWeight, kWR = FLAT ? 1 : kResidualWeight;
    const bool APPEND = FUSED && a.append;
    static_assert(!PAIRED || LO, "the paired rows are the hi and lo parts");
    constexpr int NHQ = PAIRED ? 2 : kNH;                  // heads the quantized passes work on
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
    _Float16 *ps = lds;                                    // [NCG][kNH][kPsH] halfs (quantized passes)

    const int lane = threadIdx.x;
    const int NU = a.units * a.hsets;

    // ---------------- the work list: total weight P, this wave's range, the unit that holds its start.
    // Lane l looks at units l, l+64, ...; up to 256 units the lengths stay in registers between the two
    // steps (sum, then locate), beyond that the second step reads them again.  Units without any token
    // get their zeros here.
    auto zero_fill = [&](int uu) {
        const int u = uu >> a.hs_shift, hs = uu & (a.hsets - 1);
        const int bi = (int)fast_div((uint32_t)u, a.hkv_magic, a.hkv_shift);
        const int bq0 = bi * a.Hq + (u - bi * a.Hkv) * a.rep + hs * kNH;
        const int nh = min(kNH, a.rep - hs * kNH);
        for (int i = lane; i < nh * kD; i += 64) a.out[(size_t)bq0 * kD + i] = 0;   // the whole wave
        if (APPEND && lane == 0 && hs == 0) a.r_len_out[u] = a.r_len[u];          // (nothing was appended: see res_len)
    };
    // lengths of units base + 64k + lane, k = 0..3: all eight loads go out before any is waited for
    auto lengths4 = [&](int base, int (&T)[4], int (&R)[4]) {
        int t[4], r[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int u = min(base + 64 * k + lane, NU - 1) >> a.hs_shift;
            t[k] = a.q_len[u];
            r[k] = a.r_len[u];
        }
        asm volatile("" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]));
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const bool in = base + 64 * k + lane < NU;
            T[k] = in ? clampi(t[k], 0, a.Tcap) : 0;
            R[k] = in ? res_len(APPEND, a, r[k]) : 0;
        }
    };
    auto weight_of = [&](int T, int R) -> int {
        if (APPEND) R &= (1 << kAppBit) - 1;
        return kWQ * ((T + kPass - 1) / kPass) + kWR * ((R + 63) >> 6);
    };
    const bool small = NU <= 256;
    int Tl[4], Rl[4], wl4[4], incl4[4];
    int P = 0;
    bool empties = false;                                  // some unit of this wave's share holds no token
    // Fused step: workgroup b files the new rows of units b, b + grid size, ... in the residual buffer (32 lanes,
    // 16 bytes each: the key row, then the value row).  Nothing in this launch reads those rows from the buffer
    // -- the residual items take them from the caller's arrays -- so the copy needs no ordering against the
    // rest; the first unit's rows are requested here and stored after the lengths below have arrived, so that
    // the wave waits once for both.  (Inside the residual item the copy cost the whole launch 4 us: whatever
    // form it took there, the item's local-memory reads and its loads lost their overlap.)
    uint4 new_piece = {0u, 0u, 0u, 0u};
    int new_row = -1;
    const bool files_new = APPEND && (int)blockIdx.x < a.units && lane < 32;
    auto new_src = [&](int u) { return reinterpret_cast<const uint4 *>((lane < 16 ? a.k_new : a.v_new) + (size_t)u * kD) + (lane & 15); };
    auto new_dst = [&](int u, int r) { return reinterpret_cast<uint4 *>(const_cast<uint16_t *>(lane < 16 ? a.Rk : a.Rv) + ((size_t)u * a.Rcap + r) * kD) + (lane & 15); };
    if (files_new) {
        new_row = a.r_len[blockIdx.x];
        new_piece = *new_src(blockIdx.x);
    }
    for (int base = 0; base < NU; base += 256) {
        lengths4(base, Tl, Rl);
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int uu = base + 64 * k + lane;
            wl4[k] = weight_of(Tl[k], Rl[k]);
            empties |= uu < NU && wl4[k] == 0 && uu % (int)gridDim.x == (int)blockIdx.x;
            incl4[k] = wave_scan_i32(wl4[k]);
            P += __builtin_amdgcn_readlane(incl4[k], 63);
        }
    }
    if (files_new) {
        if (new_row >= 0 && new_row < a.Rcap) *new_dst(blockIdx.x, new_row) = new_piece;
        for (int u = blockIdx.x + gridDim.x; u < a.units; u += gridDim.x) {     // (more units than workgroups)
            const int r = a.r_len[u];
            if (r >= 0 && r < a.Rcap) *new_dst(u, r) = *new_src(u);
        }
    }
    if (__ballot(empties)) {                               // rare: look again, one unit at a time
        for (int uu = blockIdx.x; uu < NU; uu += gridDim.x) {
            const UnitItems it = unit_items(APPEND, a, uu);
            if (it.nq + it.nr == 0) zero_fill(uu);
        }
    }
    // The weight line is cut into NW ranges, each at least one residual item long.  NW is a power of two so
    // that the cuts need no division.
    if (P == 0) return;
    const int nw_cap = max(1, min((int)gridDim.x, P / kWR));
    const int nw_log = 31 - __builtin_clz(nw_cap), NW = 1 << nw_log;
    if ((int)blockIdx.x >= NW) return;
    // Wave numbers.  The hardware serves the older of the two waves on a SIMD first, so the workgroups
    // that were dispatched first (they fill the first wave slot of every SIMD, a.first_slot of them) get
    // through their passes measurably faster than the rest.  When the launch fills both slots, workgroup b
    // and workgroup b + a.first_slot take the neighbouring numbers 2b and 2b + 1, so that every unit is
    // served by both kinds in equal parts and all units finish together.
    const bool paired = NW == 2 * a.first_slot;
    const int w = !paired ? (int)blockIdx.x
                : (int)blockIdx.x < a.first_slot ? 2 * (int)blockIdx.x : 2 * ((int)blockIdx.x - a.first_slot) + 1;
    // (the wave in the first slot of a SIMD runs faster; both parts of a pair range must stay longer than one
    // item, so that every wave between the first and the last of a unit owns an item of it)
    const int want16 = min(max(a.skew16, 4), 12);
    const int skew16 = paired && ((((2L * P) >> nw_log) * min(want16, 16 - want16)) >> 4) >= kWR ? want16 : 8;
    const long start = range_start(w, P, nw_log, skew16), end = range_start(w + 1, P, nw_log, skew16);
    // (NW / P as a wave-uniform value in a scalar register)
    const float inv_p = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, (float)NW / (float)P)));

    // ---------------- the unit whose weight span holds position `start`
    int up = -1;
    long ib = 0;                                           // position of the unit's first item
    int T_first = 0, R_first = 0;                          // its lengths
    {
        long running = 0;
        for (int base = 0; base < NU && up < 0; base += 256) {
            if (!small) {
                lengths4(base, Tl, Rl);
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    wl4[k] = weight_of(Tl[k], Rl[k]);
                    incl4[k] = wave_scan_i32(wl4[k]);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const long excl = running + incl4[k] - wl4[k];
                const bool hit = up < 0 && wl4[k] > 0 && start >= excl && start < excl + wl4[k];
                const unsigned long long mask = __ballot(hit);
                if (mask) {
                    const int src = __ffsll((long long)mask) - 1;
                    up = base + 64 * k + src;
                    ib = running + __builtin_amdgcn_readlane(incl4[k] - wl4[k], src);
                    T_first = __builtin_amdgcn_readlane(Tl[k], src);
                    R_first = __builtin_amdgcn_readlane(Rl[k], src);
                }
                running += __builtin_amdgcn_readlane(incl4[k], 63);
            }
        }
    }
    const int up_first = up;

    const int blk4 = lane >> 2, row = lane & 3;            // block of 4 lanes; row = query head this lane
                                                           // supplies as A operand
    const int gl = blk4 / BGK;                             // K group (of the pass) of this lane's tokens
    const int bbk = blk4 % BGK;                            // this lane's bin of k-steps: bbk, bbk+BGK, ...
    const int bbv = blk4 % BGV;                            // same on the V side (k-steps of 4 tokens)
    const int cg0 = lane / G;                              // channel groups of channels lane, lane+64
    const int cg1 = (lane + 64) / G;
    // Tokens 2*lane, 2*lane+1 are field j = lane & 7 of their V word.  The weights of this lane carry the
    // constant factor 2^lg = 16 * 4^-shift so that the masked V field needs no shift; the lane's running
    // sums l and oz carry the same factor and are unscaled once per unit.
    const float kscale = a.c1 * 16777216.0f;               // undo the 2^-24 of the subnormal code fields

    // A wave owns the items whose start position lies in [start, end).
    for (; up < NU && ib < end; up++) {
        // (the lengths of the first unit are already known)
        const UnitItems it = up == up_first ? make_items(APPEND, T_first, R_first) : unit_items(APPEND, a, up);
        const int wt = kWR * it.nr + kWQ * it.nq;
        if (wt == 0) continue;
        const long ib_next = ib + wt;
        // this wave's items of the unit (the offsets are clamped to the unit's span first, so 32-bit
        // arithmetic suffices): front residual items f0..f1-1, passes j0..j1-1, back residual items b0..b1-1
        const int nf = (it.nr + 1) >> 1, nb = it.nr >> 1;
        const int span = wt + kWR;
        const int ds = (int)min((long)span, max(0L, start - ib)), de = (int)min((long)span, max(0L, end - ib));
        const int dq = kWR * nf, db = dq + kWQ * it.nq;
        const int f0 = min(nf, (ds + kWR - 1) / kWR), f1 = min(nf, (de + kWR - 1) / kWR);
        const int j0 = min(it.nq, (max(0, ds - dq) + kWQ - 1) / kWQ), j1 = min(it.nq, (max(0, de - dq) + kWQ - 1) / kWQ);
        const int b0 = min(nb, (max(0, ds - db) + kWR - 1) / kWR), b1 = min(nb, (max(0, de - db) + kWR - 1) / kWR);
        if (f0 >= f1 && j0 >= j1 && b0 >= b1) { ib = ib_next; continue; }
        const int u = up >> a.hs_shift, hs = up & (a.hsets - 1);
        const int bi = (int)fast_div((uint32_t)u, a.hkv_magic, a.hkv_shift);
        const int bq0 = bi * a.Hq + (u - bi * a.Hkv) * a.rep + hs * kNH;
        const int nheads = min(kNH, a.rep - hs * kNH);
        const int t_end = it.T;
        // the waves that own items of this unit: from the owner of the first item to the owner of the last
        const int wf = wave_of(ib, P, nw_log, inv_p, skew16);
        const int wl = wave_of(ib_next - (nb ? kWR : it.nq ? kWQ : kWR), P, nw_log, inv_p, skew16);
        const int expected = wl - wf + 1;
        const uint32_t *Kc = a.Kc + (size_t)u * kc_words(a.Tcap);
        const uint32_t *Vc = a.Vc + (size_t)u * vc_words(a.Tcap);
        const uint16_t *Ks = a.Ks + (size_t)u * (a.Tcap / G) * kD;
        const uint16_t *Kz = a.Kz + (size_t)u * (a.Tcap / G) * kD;
        const uint16_t *Vs = a.Vs + (size_t)u * a.Tcap * NCG;
        const uint16_t *Vz = a.Vz + (size_t)u * a.Tcap * NCG;

        int lane_u = lane;
        asm volatile("" : "+v"(lane_u));                   // (opaque copy: per-lane load offsets are set up per unit)
        const int bbk_u = (lane_u >> 2) % BGK;
        // Loaders of one pass's tiles, in the pieces the phases consume them in (each piece is requested again,
        // for the wave's next pass, as soon as its registers have been read for the last time: every piece is
        // then in flight for about a whole pass, which is what keeps enough bytes outstanding per wave).
        auto load_k_meta = [&](KD &d, int tp) {
            const bool gvalid = tp + gl * G < t_end;
            const size_t go = ((size_t)(tp / G) + (gvalid ? gl : 0)) * kD + bbk_u * (NKR * 4);
            d.ks = load_words<NKW>(Ks + go);
            d.kz = load_words<NKW>(Kz + go);
        };
        auto load_k_codes = [&](KD &d, int tp, int half) {       // half 0: words 0..3 of both tokens, 1: words 4..7
            const u4 *ktile = reinterpret_cast<const u4 *>(Kc + (size_t)(tp >> 7) * 1024);
            d.kw[half] = ktile[half * 64 + lane_u];
            d.kw[2 + half] = ktile[(2 + half) * 64 + lane_u];
        };
        auto load_v_meta = [&](VD &d, int tp) {
            // past the end the (clamped) load still happens (the weights of those tokens are zero), so that the
            // number of loads in flight is the same on every path
            const bool valid = tp + 2 * lane_u < t_end;
            const size_t vo = (size_t)(valid ? tp + 2 * lane_u : tp) * NCG;
            d.vs = load_words<NCG>(Vs + vo);
            d.vz = load_words<NCG>(Vz + vo);
        };
        auto load_v_codes = [&](VD &d, int tp, int tl) {         // tl: 64-token tile of the pass
            const u4 *vtile = reinterpret_cast<const u4 *>(Vc + (size_t)(tp >> 6) * (4 * kD));
            d.vw[0][tl] = vtile[tl * kD + lane_u];
            d.vw[1][tl] = vtile[tl * kD + lane_u + 64];
        };
        auto load_k = [&](int tp) -> KD {
            KD d;
            load_k_codes(d, tp, 0);
            load_k_codes(d, tp, 1);
            load_k_meta(d, tp);
            return d;
        };
        auto load_v = [&](int tp) -> VD {
            VD d;
            load_v_codes(d, tp, 0);
            load_v_codes(d, tp, 1);
            load_v_meta(d, tp);
            return d;
        };

        // Operand ranges.  The A operands of both products are fp16: q*Ks*4^-j on the K side and p*Vs*2^lg on
        // the V side (p <= 1, 2^lg <= 2^hd).  The first attempt uses the scalings that keep the most precision
        // (q as it is, hd = 4); they hold as long as |q*Ks| < 65504 and Vs < 4096.  Beyond that an operand
        // overflows to infinity, which ends up in the wave's sums: an infinite q*Ks meets a code 0 in its group
        // (every group with a non-zero scale has one), the product is NaN, so is that token's weight, and the sum
        // of weights keeps it; an infinite p*Vs makes the output sums infinite or NaN.  The sums are checked once
        // per unit, and if one is not finite the wave does its items of the unit again with q scaled per head to
        // below 1 and hd = -1: then |A| <= max Ks, max Vs / 2 <= 43669 whatever the inputs (the largest fp16
        // scale is (65504 + 65504) / 3).  No cost for data inside the range; outside it the result keeps fewer
        // bits of the small weights.
        float m[kNH], lsum[kNH];                           // running max; sum of weights (wave-uniform at the end)
        float oa[kNH], ob[kNH];                            // un-normalised output of channels lane, lane+64
#pragma nounroll
        for (int attempt = 0; attempt < 2; attempt++) {
        const bool safe = attempt != 0;
        if (safe && lane == 0) atomicAdd(a.redo, 1);       // (diagnostics: how often the second attempt is taken)
        const float hd = safe ? -1.0f : 4.0f;
        const float lg = hd - (float)fld_shift(lane & 7);
        const float vun = safe ? 33554432.0f : 1048576.0f; // 2^24 (subnormal fields) / 2^hd (ps headroom)
        const float inv_vun = 1.0f / vun;
        // This lane's query values for the quantized passes (head `row`, the channels of its k-steps).
        h2 qraw[NKR][2];
        auto load_q = [&]() {
#pragma unroll
            for (int i = 0; i < NKR; i++) {
                const int c = 4 * (bbk_u + BGK * i);
                uint2 bits = {0u, 0u};
                const int hq = PAIRED ? (lane_u & 3) >> 1 : (lane_u & 3);   // the head whose A rows this lane supplies
                if (hq < nheads && j0 < j1) bits = *reinterpret_cast<const uint2 *>(a.q + (size_t)(bq0 + hq) * kD + c);
                qraw[i][0] = as_h2(bits.x);
                qraw[i][1] = as_h2(bits.y);
            }
        };
        // The tiles of the first pass are requested before anything else is waited for; without residual items
        // in front the query values go first (they are needed first, and a wait for them then does not wait
        // for the tiles), with residual items they are fetched afterwards (fewer registers live in between).
        KD kd = {};
        VD vd = {};
        const bool front = f0 < f1;
        if (!front) load_q();
        if (j0 < j1) {
            kd = load_k(j0 * kPass);
            vd = load_v(j0 * kPass);
        }
        // the wave's online-softmax state for this unit
        float l_lane[kNH];
        f4 O0 = {0.f, 0.f, 0.f, 0.f}, O1 = {0.f, 0.f, 0.f, 0.f};   // channel lane / lane+64, 4 heads each
        float oz[kNH][NCG];
#pragma unroll
        for (int h = 0; h < kNH; h++) {
            m[h] = -1e30f; l_lane[h] = 0.f;
#pragma unroll
            for (int g = 0; g < NCG; g++) oz[h][g] = 0.f;
        }

        // =============================== residual items (64 fp16 tokens each): Algorithm 1's R_K t_Q^T and
        // A_unquant R_V, on the same 4x4x4 matrix instruction as the quantized passes (the vector ALU is
        // several times slower here because the wave shares its SIMD with one that saturates the matrix
        // pipe).  The 64 key rows, then the 64 value rows, are fetched with fully coalesced loads (4 rows
        // per instruction, 16 lanes x 16 B per row) and staged in LDS.  Scores: lane = token, its key row
        // read back as the B operand, q as the A operand broadcast to all 16 blocks.  Values: lane =
        // channels lane, lane+64, the B operand gathered token by token from the staged rows, the weights
        // p (fp16, through LDS) as the broadcast A operand.  The result is folded into the wave's state.
        auto residual_items = [&](int lo, int hi, int odd) {   // even items sit before the passes, odd ones after
#pragma unroll 1
        for (int fi = lo; fi < hi; fi++) {
            const int ri = 2 * fi + odd;
            const int R = it.R;
            _Float16 *pr = lds;                            // [kNH][64 + 8] halfs: weights of the item's tokens
            _Float16 *rows = lds + kNH * kD;               // [64][kKRowH] halfs: key rows, then value rows
            constexpr int kPrH = 72;
            const uint16_t *Rk = a.Rk + (size_t)u * a.Rcap * kD;
            const uint16_t *Rv = a.Rv + (size_t)u * a.Rcap * kD;
            int lane_r = lane;                             // (opaque copy: keeps the address terms below out of
            asm volatile("" : "+v"(lane_r));               //  the registers that live across the pass loop)
            const int rsub = lane_r >> 4, piece = lane_r & 15;  // row within a group of 4, 16-byte piece of the row
            const int t0 = ri * 64;
            const bool valid = t0 + lane < R;

            // (fused step: the unit's last residual row is the token this launch appends; it is read from the
            // caller's new rows, never from the residual buffer, where another wave files it at some point of
            // this launch)
            const int r_new = it.rn;                       // (a full or invalid buffer takes no token)
            const uint16_t *kn = APPEND ? a.k_new + (size_t)u * kD : nullptr, *vn = APPEND ? a.v_new + (size_t)u * kD : nullptr;
            // (the rows are loaded as in the plain call; the item that holds the new row then loads it once more,
            // from the caller's array, into the registers of the four-row step it belongs to: one wave-uniform branch
            // per step instead of a select per row)
            const bool has_new = APPEND && r_new >= t0 && r_new < t0 + 64;     // (uniform)
            const int new_step = (r_new - t0) >> 2, new_sub = (r_new - t0) & 3;
            Words<64> g;
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int rr = t0 + 4 * i + rsub;
                const uint16_t *src = Rk + (size_t)(rr < R ? rr : 0) * kD;
                const uint4 x = reinterpret_cast<const uint4 *>(src)[piece];
                g.v[4 * i] = x.x; g.v[4 * i + 1] = x.y; g.v[4 * i + 2] = x.z; g.v[4 * i + 3] = x.w;
            }
            if (has_new) {
#pragma unroll
                for (int i = 0; i < 16; i++)
                    if (i == new_step && rsub == new_sub) {
                        const uint4 x = reinterpret_cast<const uint4 *>(kn)[piece];
                        g.v[4 * i] = x.x; g.v[4 * i + 1] = x.y; g.v[4 * i + 2] = x.z; g.v[4 * i + 3] = x.w;
                    }
            }
            // A operands of the scores: block b supplies k-steps b and b+16 (channels 4b.., 64+4b..) of head `row`
            h4 qa[2];
#pragma unroll
            for (int i = 0; i < 2; i++) {
                uint2 bits = {0u, 0u};
                if ((lane_r & 3) < nheads) bits = *reinterpret_cast<const uint2 *>(a.q + (size_t)(bq0 + (lane_r & 3)) * kD + 4 * ((lane_r >> 2) + 16 * i));
                const h2 lo = as_h2(bits.x), hi = as_h2(bits.y);
                qa[i] = h4{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int i = 0; i < 16; i++)
                *reinterpret_cast<uint4 *>(rows + (4 * i + rsub) * kKRowH + piece * 8) =
                    uint4{g.v[4 * i], g.v[4 * i + 1], g.v[4 * i + 2], g.v[4 * i + 3]};
            // the value rows are requested now and travel while the scores are computed
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int rr = t0 + 4 * i + rsub;
                const uint16_t *src = Rv + (size_t)(rr < R ? rr : 0) * kD;
                const uint4 x = reinterpret_cast<const uint4 *>(src)[piece];
                g.v[4 * i] = x.x; g.v[4 * i + 1] = x.y; g.v[4 * i + 2] = x.z; g.v[4 * i + 3] = x.w;
            }
            if (has_new) {
#pragma unroll
                for (int i = 0; i < 16; i++)
                    if (i == new_step && rsub == new_sub) {
                        const uint4 x = reinterpret_cast<const uint4 *>(vn)[piece];
                        g.v[4 * i] = x.x; g.v[4 * i + 1] = x.y; g.v[4 * i + 2] = x.z; g.v[4 * i + 3] = x.w;
                    }
            }
            __builtin_amdgcn_wave_barrier();

            f4 sc = {0.f, 0.f, 0.f, 0.f};                  // scores of token t0 + lane for the 4 heads
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const u4 kk = *reinterpret_cast<const u4 *>(rows + lane * kKRowH + i * 8);   // channels 8i..8i+7
                const h2 k0 = as_h2(kk[0]), k1 = as_h2(kk[1]), k2 = as_h2(kk[2]), k3 = as_h2(kk[3]);
                mfma_bc<4>(sc, qa[(2 * i) / 16], h4{k0[0], k0[1], k1[0], k1[1]}, (2 * i) % 16);
                mfma_bc<4>(sc, qa[(2 * i + 1) / 16], h4{k2[0], k2[1], k3[0], k3[1]}, (2 * i + 1) % 16);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 16; i++)
                *reinterpret_cast<uint4 *>(rows + (4 * i + rsub) * kKRowH + piece * 8) =
                    uint4{g.v[4 * i], g.v[4 * i + 1], g.v[4 * i + 2], g.v[4 * i + 3]};

            // softmax update against the wave's state
            float s[kNH], mn[kNH];
            bool grow = false;
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                s[h] = valid ? sc[h] * a.c1 : -INFINITY;
                mn[h] = s[h];
            }
            wave_max64x4(mn);
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                mn[h] = fmaxf(m[h], mn[h]);
                grow |= mn[h] > m[h];
            }
            if (grow) {                                    // wave-uniform
#pragma unroll
                for (int h = 0; h < kNH; h++) {
                    const float so = fast_exp2(m[h] - mn[h]);
                    l_lane[h] *= so;
                    O0[h] *= so;
                    O1[h] *= so;
#pragma unroll
                    for (int gq = 0; gq < NCG; gq++) oz[h][gq] *= so;
                    m[h] = mn[h];
                }
            }
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                const float p = fast_exp2(s[h] - m[h]);    // 0 past the end
                l_lane[h] += p * fast_exp2(lg);            // the lane sums carry the factor 2^lg
                pr[h * kPrH + lane] = (_Float16)p;
            }
            __builtin_amdgcn_wave_barrier();

            // values: 16 k-steps of 4 tokens; block b supplies the weights of k-step b
            const h4 pa = *reinterpret_cast<const h4 *>(pr + row * kPrH + 4 * blk4);
            f4 R0 = {0.f, 0.f, 0.f, 0.f}, R1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 16; ks++) {
                const _Float16 *v = rows + (4 * ks) * kKRowH + lane;
                const h4 b0 = {v[0], v[kKRowH], v[2 * kKRowH], v[3 * kKRowH]};
                const h4 b1 = {v[64], v[kKRowH + 64], v[2 * kKRowH + 64], v[3 * kKRowH + 64]};
                mfma_bc<4>(R0, pa, b0, ks);
                mfma_bc<4>(R1, pa, b1, ks);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                O0[h] += R0[h] * inv_vun;                  // the state's outputs carry the factor 1/vun
                O1[h] += R1[h] * inv_vun;
            }
        }
        };
        if (front) {
            residual_items(f0, f1, 0);
            load_q();
        }
        {
        // =============================== quantized passes
            // the query values pre-scaled by the 4^-j of the code field (channel pair (c, c+1), c even, is field
            // (c % 16) / 2 of its K word)
            h2 qscl[NKR][2];
            // qf: the power of two this lane's head is scaled by (1 on the first attempt; on the second
            // 2^(14 - E) with E the biased exponent of the head's largest |q|, so that |q| * qf < 1)
            float qf = 1.0f;
            if (safe) {
                typedef unsigned short us2 __attribute__((ext_vector_type(2)));
                us2 mx2 = {0, 0};
#pragma unroll
                for (int i = 0; i < NKR; i++)
#pragma unroll
                    for (int ep = 0; ep < 2; ep++)
                        mx2 = __builtin_elementwise_max(mx2, __builtin_bit_cast(us2, as_u32(qraw[i][ep]) & 0x7fff7fffu));
                int mx = max((int)mx2[0], (int)mx2[1]);
                for (int d = 4; d < 64; d <<= 1) mx = max(mx, __shfl_xor(mx, d));   // lanes with the same `row`
                qf = fast_exp2(14.0f - (float)min(mx >> 10, 30));
            }
            float ksc[kNH];                                // kscale / qf of head h (wave-uniform)
#pragma unroll
            for (int h = 0; h < NHQ; h++) {
                const float f = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, qf), PAIRED ? 2 * h : h));
                ksc[h] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, kscale / f)));
            }
#pragma unroll
            for (int i = 0; i < NKR; i++) {
                const int c = 4 * (bbk + BGK * i);
#pragma unroll
                for (int ep = 0; ep < 2; ep++)
                    qscl[i][ep] = qraw[i][ep] * (_Float16)(fld_scale(((c + 2 * ep) & 15) >> 1) * qf);
            }

            float s0[kNH], s1[kNH];                        // scores of the lane's two tokens (NHQ heads)

            // ---------------- K phase: scores of tokens 2*lane, 2*lane+1 for the 4 heads
            auto k_phase = [&](KD &d, int tp, int t2) {        // t2: the pass whose tiles are requested meanwhile
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
                    if constexpr (PAIRED) {                 // odd rows carry the lo part
                        const h2 u0 = (row & 1) ? lo[0] : hi[0], u1 = (row & 1) ? lo[1] : hi[1];
                        a_hi[i] = h4{u0[0], u0[1], u1[0], u1[1]};
                    } else {
                        a_hi[i] = h4{hi[0][0], hi[0][1], hi[1][0], hi[1][1]};
                        if constexpr (LO) a_lo[i] = h4{lo[0][0], lo[0][1], lo[1][0], lo[1][1]};
                    }
                }
                __builtin_amdgcn_sched_barrier(0);         // (all A operands first: the rows are then free)
                load_k_meta(d, t2);                        // the scale / zero rows have been consumed
                __builtin_amdgcn_sched_barrier(0);
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
                        if constexpr (LO && !PAIRED) mfma_k<CBK>(acc0, acc1, a_lo[s / BGK], b0, b1, s % BGK);
                    }
                    if (wd == 3) {                         // words 0..3 are done
                        __builtin_amdgcn_sched_barrier(0);
                        load_k_codes(d, t2, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                load_k_codes(d, t2, 1);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (PAIRED) {
                    const float zz[2] = {quad_bcast<0>(qz) * a.c1, quad_bcast<2>(qz) * a.c1};
#pragma unroll
                    for (int h = 0; h < 2; h++) {
                        s0[h] = valid ? (acc0[2 * h] + acc0[2 * h + 1]) * ksc[h] + zz[h] : -INFINITY;
                        s1[h] = valid ? (acc1[2 * h] + acc1[2 * h + 1]) * ksc[h] + zz[h] : -INFINITY;
                    }
                } else {
                    const float zz[kNH] = {quad_bcast<0>(qz) * a.c1, quad_bcast<1>(qz) * a.c1,
                                           quad_bcast<2>(qz) * a.c1, quad_bcast<3>(qz) * a.c1};
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        s0[h] = valid ? acc0[h] * ksc[h] + zz[h] : -INFINITY;
                        s1[h] = valid ? acc1[h] * ksc[h] + zz[h] : -INFINITY;
                    }
                }
            };

            // ---------------- softmax update, ps table, V products
            auto v_phase = [&](VD &d, int tp, int t2) {
                const bool valid = tp + 2 * lane < t_end;
                float mn[kNH];
                bool grow = false;
#pragma unroll
                for (int h = 0; h < NHQ; h++) mn[h] = fmaxf(s0[h], s1[h]);
                if constexpr (PAIRED) wave_max64x2(mn); else wave_max64x4(mn);
#pragma unroll
                for (int h = 0; h < NHQ; h++) {
                    mn[h] = fmaxf(m[h], mn[h]);
                    grow |= mn[h] > m[h];
                }
                if (grow) {                                // wave-uniform
#pragma unroll
                    for (int h = 0; h < NHQ; h++) {
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
                    __builtin_amdgcn_sched_barrier(0);
                    load_v_meta(d, t2);                    // the scales and zero-points have been consumed
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int h = 0; h < NHQ; h++) {
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
                    if (blk == 3) {                        // the first 64-token tile is done
                        __builtin_amdgcn_sched_barrier(0);
                        load_v_codes(d, t2, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                load_v_codes(d, t2, 1);
                __builtin_amdgcn_wave_barrier();
            };

            // Every piece of a pass's tiles is requested for the next pass right after its last use and is
            // issued on every path (the last pass requests its own tiles again), so the number in flight is
            // always the same.
            for (int jj = j0; jj < j1; jj++) {
                const int tp = jj * kPass;
                const int t2 = (jj + 1 < j1 ? jj + 1 : jj) * kPass;
                k_phase(kd, tp, t2);
                v_phase(vd, tp, t2);
            }
        }
        residual_items(b0, b1, 1);

        {
            // finish: undo operand scalings, add the zero-point term
            const float unlg = fast_exp2(-lg);
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
        }
        {
            // any overflowed operand has left an infinity or a NaN in one of the sums (of the heads in use:
            // with paired rows the accumulators of rows 2 and 3 hold nothing meaningful)
            float chk = 0.f;
#pragma unroll
            for (int h = 0; h < NHQ; h++) chk += (O0[h] + O1[h]) + l_lane[h];
            if (__ballot(!(chk - chk == 0.f)) == 0) break;
        }
        }   // attempt

        // =============================== publish this wave's partial of the unit
        int lane_p = lane;
        asm volatile("" : "+v"(lane_p));                   // (opaque copy: address terms computed here, not hoisted)
        // (fused step: the unit's residual length after the append, for the next call -- into an array of its own,
        // because every wave of THIS launch still reads the old lengths when it starts; written by the wave that
        // writes the unit's output)
        auto write_next_len = [&]() {
            if (APPEND && lane == 0) a.r_len_out[u] = it.rn >= 0 ? it.rn + 1 : a.r_len[u];
        };
        if (expected == 1) {
            // the only partial of its unit: normalise and write the result directly
            write_next_len();
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                if (h < nheads) {
                    const float inv = lsum[h] > 0.f ? 1.0f / lsum[h] : 0.f;
                    a.out[(size_t)(bq0 + h) * kD + lane_p] = __half_as_ushort(__float2half_rn(oa[h] * inv));
                    a.out[(size_t)(bq0 + h) * kD + lane_p + 64] = __half_as_ushort(__float2half_rn(ob[h] * inv));
                }
            }
        } else {
            // Two-level merge.  The waves of the unit form sub-groups of 16 (by their place in the group);
            // the last partial to arrive in a sub-group merges it -- the slots are consecutive, every
            // address is a wave-uniform base plus constants, one round trip -- and, when the unit has more
            // than one sub-group, writes the result over the sub-group's first slot and takes a ticket at
            // the unit; the last sub-group to arrive merges those (slots 16 apart).  So a unit served by
            // hundreds of waves still ends with two short merges, and the first level runs while other
            // waves are still at work.
            constexpr int kSlotB = kNH * kPartialStride * 4, kHeadB = kPartialStride * 4;
            // The merging wave holds, per lane, 4 consecutive channels of two heads: lanes 0..31 of heads 0 and 2,
            // lanes 32..63 of heads 1 and 3.  One 128-bit load per lane then fetches a partial's outputs of two heads,
            // so the 16 partials of a sub-group are 32 + 4 loads: a wave can have 63 memory instructions outstanding,
            // and with 64-bit loads (68 of them) the last ones went out only after the first had returned -- two
            // round trips where this is one.
            const int half_p = lane_p >> 5, c4 = lane_p & 31;
            const unsigned lane_off = (unsigned)(half_p * kHeadB + 16 + c4 * 16);
            float M[kNH], L[kNH];
            f4 Oq[2];                                      // Oq[j]: channels 4*c4 .. 4*c4+3 of head 2*j + half_p
            // merges `count` partials, `stride` slots apart from slot `first`, into (M, L, Oq): lane s fetches
            // (max, sum) of partial s, which gives every partial's weight; the output vectors of up to 16
            // partials are requested in the same round trip (device-scope loads: sc1)
            auto merge = [&](int first, int stride, int count) {
                const char *const sbase = reinterpret_cast<const char *>(slot_ptr(a, first, 0));
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(sbase), 0, 0x7fffffff, 0x00020000);
                const unsigned step = (unsigned)stride * kSlotB;
#pragma unroll
                for (int h = 0; h < kNH; h++) { M[h] = -1e30f; L[h] = 0.f; }
                Oq[0] = f4{0.f, 0.f, 0.f, 0.f}; Oq[1] = Oq[0];
                constexpr int MB = 16;
                constexpr int kSc1 = 16;                   // cache policy of the buffer load: device scope
#pragma unroll 1
                for (int base = 0; base < count; base += MB) {
                    const int cnt = min(MB, count - base);
                    const bool has = lane < cnt;
                    const char *const mine_p = sbase + (size_t)(base + (has ? lane : 0)) * step;
                    float ms[kNH], ls[kNH], cm[kNH];
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float2 ml = ld_agent2(reinterpret_cast<const float *>(mine_p + h * kHeadB));
                        const bool on = has && h < nheads;
                        ms[h] = on ? ml.x : -1e30f;        // partials that do not exist get weight 0 below
                        ls[h] = on ? ml.y : 0.f;
                    }
                    f4 x[MB][2];
#pragma unroll
                    for (int k = 0; k < MB; k++) {
                        const unsigned pk = (unsigned)(base + min(k, cnt - 1)) * step;   // uniform
#pragma unroll
                        for (int j = 0; j < 2; j++) {
                            typedef unsigned int u4v __attribute__((ext_vector_type(4)));
                            const u4v v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, pk + (unsigned)(2 * j * kHeadB), kSc1);
                            x[k][j] = __builtin_bit_cast(f4, v);
                        }
                    }
#pragma unroll
                    for (int h = 0; h < kNH; h++) cm[h] = ms[h];
                    wave_max64x4(cm);
                    float wgt[kNH], lw[kNH];
                    float so2[2];
#pragma unroll
                    for (int h = 0; h < kNH; h++) {
                        const float Mn = fmaxf(M[h], cm[h]);
                        const float so = fast_exp2(M[h] - Mn);
                        wgt[h] = fast_exp2(ms[h] - Mn);    // exactly 0 for ms = -1e30
                        lw[h] = ls[h] * wgt[h];
                        L[h] *= so;
                        if ((h & 1) == 0) so2[h >> 1] = so; else so2[h >> 1] = half_p ? so : so2[h >> 1];
                        M[h] = Mn;
                    }
                    Oq[0] *= so2[0]; Oq[1] *= so2[1];
                    wave_sum64x4(lw);
#pragma unroll
                    for (int h = 0; h < kNH; h++) L[h] += lw[h];
#pragma unroll
                    for (int k = 0; k < MB; k++)
#pragma unroll
                        for (int j = 0; j < 2; j++) {
                            const float w0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wgt[2 * j]), k));
                            const float w1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wgt[2 * j + 1]), k));
                            const float wl = half_p ? w1 : w0;
                            Oq[j] += x[k][j] * wl;
                        }
                }
            };
            auto write_out = [&]() {
                write_next_len();
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    const int h = 2 * j + half_p;
                    if (h >= nheads) continue;
                    const float Lh = half_p ? L[2 * j + 1] : L[2 * j];
                    const float inv = Lh > 0.f ? 1.0f / Lh : 0.f;
                    const h2 r0 = {(_Float16)(Oq[j][0] * inv), (_Float16)(Oq[j][1] * inv)};
                    const h2 r1 = {(_Float16)(Oq[j][2] * inv), (_Float16)(Oq[j][3] * inv)};
                    *reinterpret_cast<uint2 *>(a.out + (size_t)(bq0 + h) * kD + 4 * c4) = uint2{as_u32(r0), as_u32(r1)};
                }
            };
            auto take_ticket = [&](int *counter) -> int {           // after this wave's stores are acknowledged
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                int old = 0;
                if (lane == 0) old = atomicAdd(counter, 1);
                return __builtin_amdgcn_readfirstlane(old);
            };

            const int me = w - wf, sg = me >> 4;
            const int n1 = min(16, expected - 16 * sg), nsg = (expected + 15) >> 4;
            const int slot1 = wf + 16 * sg + 2 * up;               // first slot of the sub-group
            const int slot = w + 2 * up;
#pragma unroll
            for (int h = 0; h < kNH; h++) {
                if (h < nheads) {
                    float *pp = slot_ptr(a, slot, h);
                    st_agent(pp + 4 + lane, oa[h]);
                    st_agent(pp + 4 + lane + 64, ob[h]);
                    if (lane == 0) { st_agent(pp, m[h]); st_agent(pp + 1, lsum[h]); }
                }
            }
            const int old1 = take_ticket(a.cnt1 + slot1);
            if (old1 == n1 - 1) {
                merge(slot1, 1, n1);
                if (lane == 0) st_agent_i32(a.cnt1 + slot1, 0);   // ready for the next call
                if (nsg == 1) {
                    write_out();
                } else {
#pragma unroll
                    for (int j = 0; j < 2; j++) {
                        const int h = 2 * j + half_p;
                        if (h < nheads) {
                            float *pp = slot_ptr(a, slot1, h) + 4 + 4 * c4;
#pragma unroll
                            for (int e = 0; e < 4; e++) st_agent(pp + e, Oq[j][e]);
                        }
                    }
#pragma unroll
                    for (int h = 0; h < kNH; h++)
                        if (h < nheads && lane == 0) { float *pp = slot_ptr(a, slot1, h); st_agent(pp, M[h]); st_agent(pp + 1, L[h]); }
                    const int old2 = take_ticket(a.cnt + up);
                    if (old2 == nsg - 1) {
                        merge(wf + 2 * up, 16, nsg);
                        write_out();
                        if (lane == 0) st_agent_i32(a.cnt + up, 0);
                    }
                }
            }
        }
        ib = ib_next;
    }
}

template <int G, bool LO, bool PAIRED, bool APPEND, bool FLAT>
static int launch_stream_w(DecArgs a, long nw, int resident, size_t lds_bytes, hipStream_t st)
{
    a.first_slot = resident / 2;
    a.skew16 = kSkew16;
    hipLaunchKernelGGL((decode_stream_kernel<G, LO, PAIRED, APPEND, FLAT>), dim3((unsigned)nw), dim3(64), lds_bytes, st, a);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

static std::atomic<int> g_decode_weights{0};
bool set_decode_weights(int mode)
{
    if (mode < 0 || mode > 2) return false;
    g_decode_weights.store(mode);
    return true;
}

template <int G, bool LO, bool PAIRED, bool APPEND>
static int launch_stream(DecArgs a, hipStream_t st)
{
    constexpr int NCG = kD / G;
    constexpr size_t q_bytes = (size_t)NCG * kPsG * 2;
    constexpr size_t r_bytes = (size_t)kNH * kD * 2 + (size_t)64 * kKRowH * 2;
    constexpr size_t lds_bytes = q_bytes > r_bytes ? q_bytes : r_bytes;
    auto kern = decode_stream_kernel<G, LO, PAIRED, APPEND, false>;
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
    // (unit weights when the launch cannot hold more items than half the waves the device holds: measured on
    // shapes of 80 to 2240 items, they win up to 608 items -- 13.3 against 16.7 us -- tie at 560 and lose from
    // 1120 on -- 19.8 against 17.7 us)
    const int mode = g_decode_weights.load();
    return (mode == 0 ? cap_items * 2 <= (long)resident : mode == 2) ? launch_stream_w<G, LO, PAIRED, APPEND, true>(a, nw, resident, lds_bytes, st)
                                 : launch_stream_w<G, LO, PAIRED, APPEND, false>(a, nw, resident, lds_bytes, st);
}

template <bool LO, bool PAIRED>
static int launch_stream_g(const DecArgs &a, int G, hipStream_t st)
{
    if (a.append) {
        switch (G) {
        case 16: return launch_stream<16, LO, PAIRED, true>(a, st);
        case 32: return launch_stream<32, LO, PAIRED, true>(a, st);
        case 64: return launch_stream<64, LO, PAIRED, true>(a, st);
        case 128: return launch_stream<128, LO, PAIRED, true>(a, st);
        }
        return MINIKV_EUNSUPPORTED;
    }
    switch (G) {
    case 16: return launch_stream<16, LO, PAIRED, false>(a, st);
    case 32: return launch_stream<32, LO, PAIRED, false>(a, st);
    case 64: return launch_stream<64, LO, PAIRED, false>(a, st);
    case 128: return launch_stream<128, LO, PAIRED, false>(a, st);
    }
    return MINIKV_EUNSUPPORTED;
}

int launch_decode_tiled(const DecArgs &a, int G, int units, int variant, hipStream_t st)
{
    (void)units;
    if (variant != 3) return MINIKV_EINVAL;
    return a.rep <= 2 ? launch_stream_g<true, true>(a, G, st) : launch_stream_g<true, false>(a, G, st);
}

}  // namespace minikv
