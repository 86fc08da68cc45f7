// Token selection at the end of the prefill (Section 3.1.2, Algorithm 1 line 3): per unit keep the recent
// window and, of the other prompt tokens, the n_hh with the largest cumulative attention score; write the
// kept positions in ascending order.
//
// Two kernels.
//   score_key_kernel   (only when a unit has several query heads) streams the rep fp32 score rows of a
//                      unit once, adds them in head order in fp32 and stores an order-preserving 32-bit
//                      key per token.  Grid over (unit, 4096-token chunk): the whole chip streams.
//   select_kernel      one workgroup of 16 waves per unit.  A radix select (digits of 11, 11 and 10 bits of the
//                      key from the top; LDS histogram, scan from the top bin down; the first digit is counted
//                      while the keys are read from memory) finds the key T of the weakest kept heavy hitter
//                      and how many tokens equal to T are kept; then one ordered compaction
//                      pass writes position i if key_i > T, or key_i == T and fewer than that many equal
//                      keys precede it, to slot (#larger before i) + min(#equal before i, kept equals).
//                      Equal scores therefore go to the earlier position and the output is ascending
//                      without a sort.  When the prompt fits, the keys are read from memory once and held
//                      in LDS (up to 32768 tokens = 128 KB) for the other passes.
#include "common.h"

#include <atomic>

namespace minikv {

constexpr int kSelThreads = 1024;      // 16 waves: one workgroup per unit
constexpr int kSelBins = 2048;         // 11-bit digits
constexpr int kSelLoads = 8;           // keys per thread in flight in a histogram pass
constexpr int kSelSparse = 56;         // of a wave's 64 lanes with 8 keys each in such a step: matches in up to this
                                       // many lanes count as few
constexpr int kSelRangeLoads = 16;     // ... and in the first pass, which streams them from memory
constexpr int kSelFixedWords = kSelBins + 2 * 16 + 16 + 16;   // hist, compaction totals (two buffers), scan totals, result
constexpr int kSelMaxCached = 32768;   // most keys held in LDS

// Order-preserving map from finite floats to unsigned integers; the two zeros map to one key.
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// REP > 0: query heads per unit known at compile time, so that all REP x 4 loads of a step are in flight
// together; REP == 0: any number of heads, one load at a time.
template <int REP>
__global__ __launch_bounds__(256) void score_key_kernel(const float *__restrict__ A, uint32_t *__restrict__ keys,
                                                        int rep_rt, long L, int nchunk)
{
    const int rep = REP ? REP : rep_rt;
    const long unit = blockIdx.x / nchunk;
    const long base = (long)(blockIdx.x % nchunk) * 4096;
    const float *rows = A + unit * rep * L;
    for (int e0 = 0; e0 < 16; e0 += 4) {
        float s[4];
        if (REP) {
            float x[4][REP ? REP : 1];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long i = min(base + (e0 + e) * 256 + (long)threadIdx.x, L - 1);   // clamped: no branch at the loads
#pragma unroll
                for (int h = 0; h < REP; ++h) x[e][h] = rows[h * L + i];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s[e] = x[e][0];
#pragma unroll
                for (int h = 1; h < REP; ++h) s[e] = s[e] + x[e][h];                   // head order, one rounding per add
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long i = min(base + (e0 + e) * 256 + (long)threadIdx.x, L - 1);
                s[e] = rows[i];
                for (int h = 1; h < rep; ++h) s[e] = s[e] + rows[h * L + i];
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long i = base + (e0 + e) * 256 + threadIdx.x;
            if (i < L) keys[unit * L + i] = score_key(s[e]);
        }
    }
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves only (no LDS traffic):
// shifts by 1, 2, 3 inside each row of 16 lanes, then by 4 and 8 on the lanes that have such a neighbour, then
// lane 15 of a row into the next row and lane 31 into the upper half.  A lane a move does not reach adds 0.
__device__ __forceinline__ int wave_scan_incl(int v)
{
    int s = v;
    s += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);     // row_shr:1
    s += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);     // row_shr:2
    s += __builtin_amdgcn_update_dpp(0, v, 0x113, 0xf, 0xf, true);     // row_shr:3
    s += __builtin_amdgcn_update_dpp(0, s, 0x114, 0xf, 0xe, true);     // row_shr:4, lanes 4..15 of a row
    s += __builtin_amdgcn_update_dpp(0, s, 0x118, 0xf, 0xc, true);     // row_shr:8, lanes 8..15 of a row
    s += __builtin_amdgcn_update_dpp(0, s, 0x142, 0xa, 0xf, false);    // row_bcast:15 into rows 1 and 3
    s += __builtin_amdgcn_update_dpp(0, s, 0x143, 0xc, 0xf, false);    // row_bcast:31 into rows 2 and 3
    return s;
}

// One more count for digit d from every lane with match set.  The lanes that share the first matching lane's
// digit are counted with one ballot and added once (constant or heavily tied scores would otherwise queue
// on one LDS address); the others add one each.
__device__ __forceinline__ void hist_add(int *hist, bool match, int d, int lane)
{
    const unsigned long long m = __ballot(match);
    if (m == 0) return;
    const int first = __ffsll((long long)m) - 1;
    const int d0 = __shfl(d, first, 64);
    const unsigned long long same = __ballot(match && d == d0);
    if (lane == first)
        atomicAdd(&hist[d0], (int)__popcll(same));
    else if (match && d != d0)
        atomicAdd(&hist[d], 1);
}

// FROM_FLOAT: the scores are read from A (REP rows per unit, added in head order in binary32 while they are read;
// with REP > 1 only when the keys then stay in LDS), else the keys score_key_kernel left in `keys`.
template <bool FROM_FLOAT, int REP = 1>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float *__restrict__ A,
                                                             const uint32_t *__restrict__ keys, long L,
                                                             const int *__restrict__ n_hh,
                                                             const int *__restrict__ n_rw,
                                                             int *__restrict__ idx, long idx_stride,
                                                             int *__restrict__ n_tok, int cached)
{
    extern __shared__ __align__(16) uint32_t smem[];
    int *hist = (int *)smem;                         // [kSelBins]
    int *sub_tot = hist + kSelBins;                  // [2][16]
    int *scan_tot = sub_tot + 2 * 16;                // [16]
    int *found = scan_tot + 16;                      // [3] digit, kept count below it, keys in the digit's bin
    uint32_t *ck = smem + kSelFixedWords;            // [L] when cached

    const long u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = __builtin_amdgcn_readfirstlane(wave);             // the same number, known to be wave-uniform
    const long rw = n_rw[u], hh = n_hh[u];
    if (rw < 0 || hh < 0 || rw > L || hh > L - rw || hh + rw > idx_stride) {
        if (tid == 0) n_tok[u] = 0;
        return;
    }
    const int N = (int)(L - rw), k = (int)hh;
    int *row = idx + u * idx_stride;
    for (int j = tid; j < (int)rw; j += kSelThreads) row[k + j] = N + j;          // the recent window
    if (tid == 0) n_tok[u] = k + (int)rw;
    if (k == 0) return;
    if (k == N) {
        for (int j = tid; j < N; j += kSelThreads) row[j] = j;
        return;
    }
    const float *arow = A + u * REP * L;
    const uint32_t *krow = keys + u * L;
    // raw 32 bits of token i, and the key they stand for
    auto gload = [&](int i) -> uint32_t { return FROM_FLOAT ? __float_as_uint(arow[i]) : krow[i]; };
    auto gkey = [&](uint32_t raw) -> uint32_t { return FROM_FLOAT ? score_key(__uint_as_float(raw)) : raw; };
    // keys of tokens start .. start+3 (start a multiple of 4); tokens at or beyond N give unspecified values
    const int npad = (N + 3) & ~3;
    auto load4 = [&](int start, uint32_t *out) {
        if (cached) {
            const uint4 q = *(const uint4 *)&ck[min(start, npad - 4)];
            out[0] = q.x, out[1] = q.y, out[2] = q.z, out[3] = q.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = gload(min(start + j, N - 1));
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = gkey(out[j]);
        }
    };

    // ---- radix select on the key, 11 + 11 + 10 bits from the top.  Bits hi and above of T are known (`prefix`);
    // `rem` = how many tokens sharing them are still to be kept.  The FIRST digit is counted while the keys are
    // read from memory (and go to LDS when they fit): that pass waits for memory, the LDS counting rides along.
    uint32_t prefix = 0;
    int rem = k, in_bin = 0;                             // (in_bin: after the last digit, the keys equal to T)
    int hi = 32;
    // bins from the top down, two per thread; the thread whose pair crosses `rem` owns the digit
    auto settle_digit = [&](int lo) {
        const int c0 = hist[kSelBins - 1 - 2 * tid], c1 = hist[kSelBins - 2 - 2 * tid];
        int incl = wave_scan_incl(c0 + c1);
        if (lane == 63) scan_tot[wave] = incl;
        __syncthreads();
        {
            const int t = lane < 16 ? scan_tot[lane] : 0;              // totals of the 16 waves, one read
            const int ti = wave_scan_incl(t);
            incl += __builtin_amdgcn_readlane(ti, wv) - __builtin_amdgcn_readlane(t, wv);   // waves before mine
        }
        const int excl = incl - c0 - c1;
        if (excl < rem && rem <= incl) {
            const bool upper = excl + c0 >= rem;
            found[0] = kSelBins - 1 - 2 * tid - (upper ? 0 : 1);
            found[1] = rem - (upper ? excl : excl + c0);
            found[2] = upper ? c0 : c1;
        }
        __syncthreads();
        prefix |= (uint32_t)found[0] << lo;
        rem = found[1];
        in_bin = found[2];
        hi = lo;
        __syncthreads();
    };
    for (int b = tid; b < kSelBins; b += kSelThreads) hist[b] = 0;
    __syncthreads();
    constexpr int NT = kSelRangeLoads / REP;             // tokens per thread and step: kSelRangeLoads loads in flight
    for (int base = 0; base < N; base += kSelThreads * NT) {
        uint32_t kk[NT];
        // every load of the step is issued before the first is used: indices clamped, no branches
        if (REP == 1) {
#pragma unroll
            for (int e = 0; e < NT; ++e) kk[e] = gload(min(base + e * kSelThreads + tid, N - 1));
#pragma unroll
            for (int e = 0; e < NT; ++e) kk[e] = gkey(kk[e]);
        } else {
            float x[NT][REP];
#pragma unroll
            for (int e = 0; e < NT; ++e)
#pragma unroll
                for (int h = 0; h < REP; ++h) x[e][h] = arow[h * L + min(base + e * kSelThreads + tid, N - 1)];
#pragma unroll
            for (int e = 0; e < NT; ++e) {
                float sum = x[e][0];
#pragma unroll
                for (int h = 1; h < REP; ++h) sum = sum + x[e][h];                          // head order, one rounding per add
                kk[e] = score_key(sum);
            }
        }
#pragma unroll
        for (int e = 0; e < NT; ++e) {
            const int i = base + e * kSelThreads + tid;
            if (cached && i < N) ck[i] = kk[e];
            hist_add(hist, i < N, (int)(kk[e] >> 21), lane);
        }
    }
    __syncthreads();
    settle_digit(21);
    // Further digits are needed only while the bin of the cut holds more keys than are kept from it.  Once ALL of
    // them are kept (typically after the second digit: 32768 keys over four million bins leave the weakest kept
    // key alone in its bin), T = the bin's lowest key does the same job, "kept" being key >= T.  (Only with the
    // keys in LDS: the compaction that re-reads them from memory keeps the exact T.)
    while (hi > 0 && !(cached && in_bin == rem)) {
        const int lo = max(hi - 11, 0);
        const uint32_t dm = (1u << (hi - lo)) - 1u;
        for (int b = tid; b < kSelBins; b += kSelThreads) hist[b] = 0;
        __syncthreads();
        for (int base = 0; base < N; base += kSelThreads * kSelLoads) {
            // slot e of this thread holds token tok(e): from LDS two runs of 4 consecutive tokens (128-bit
            // reads), from memory consecutive lanes take consecutive tokens (coalesced); any order will do here
            uint32_t kk[kSelLoads];
            auto tok = [&](int e) {
                return cached ? base + ((e >> 2) * kSelThreads + tid) * 4 + (e & 3) : base + e * kSelThreads + tid;
            };
            if (cached) {
#pragma unroll
                for (int g = 0; g < kSelLoads / 4; ++g) load4(tok(4 * g), &kk[4 * g]);
            } else {
#pragma unroll
                for (int e = 0; e < kSelLoads; ++e) kk[e] = gload(min(tok(e), N - 1));
#pragma unroll
                for (int e = 0; e < kSelLoads; ++e) kk[e] = gkey(kk[e]);
            }
            bool match[kSelLoads];
            unsigned long long lanes = 0;              // lanes that hold a token still sharing the prefix
            const uint32_t span = hi < 32 ? 1u << hi : 0u;           // (hi < 32 here: the first digit is settled)
            if (base + kSelThreads * kSelLoads <= N) { // (uniform) all but the last step: every slot is a token
#pragma unroll
                for (int e = 0; e < kSelLoads; ++e) {
                    match[e] = (kk[e] ^ prefix) < span;
                    lanes |= __ballot(match[e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < kSelLoads; ++e) {
                    match[e] = tok(e) < N && (kk[e] ^ prefix) < span;
                    lanes |= __ballot(match[e]);
                }
            }
            if (lanes == 0) continue;                  // after the first digit few tokens still share the prefix
            if (__popcll(lanes) <= kSelSparse) {
                // ... and those few spread over the bins: one plain LDS add each costs a fraction of the
                // ballots and shuffles of hist_add (5.4 -> 1.5 us for the second digit of 32768 keys)
#pragma unroll
                for (int e = 0; e < kSelLoads; ++e)
                    if (match[e]) atomicAdd(&hist[(kk[e] >> lo) & dm], 1);
            } else {
                // many: ties or a narrow range of scores, which would queue on few LDS addresses
#pragma unroll
                for (int e = 0; e < kSelLoads; ++e) hist_add(hist, match[e], (int)((kk[e] >> lo) & dm), lane);
            }
        }
        __syncthreads();
        settle_digit(lo);
    }

    // ---- ordered compaction
    const uint32_t T = prefix;
    if (cached) {
        // Keys in LDS (at most kSelMaxCached of them, so at most 8 steps of 4096 tokens): every thread counts its 4
        // consecutive tokens of every step first -- one wave scan per step, no barrier --, the 8 x 16 wave totals
        // (in token order: step, then wave) are exchanged ONCE, and then every thread knows the slots of its
        // tokens.  (One barrier per step, as in the loop below, made this phase 7 of the kernel's 26 us.)
        constexpr int NS = kSelMaxCached / (kSelThreads * 4);
        uint32_t *tots = (uint32_t *)hist;             // [NS][16] packed counts: larger | equal << 16 (each < 65536)
        uint32_t before[NS];                           // counts of the lanes before this one in its wave, per step
        const int nsteps = (N + kSelThreads * 4 - 1) / (kSelThreads * 4);
        // When every key of T's bin is kept (the usual case: no tie across the cut), "kept" is just key >= T and
        // the bookkeeping of the equal ones falls away (3.7 instead of 5.9 us on 32768 tokens).
        const bool all_equal_kept = in_bin == rem;     // (uniform)
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            before[st] = 0;
            if (st < nsteps) {                         // (uniform)
                const int start = st * kSelThreads * 4 + tid * 4;
                uint32_t key[4];
                load4(start, key);
                uint32_t tot = 0;
                if (all_equal_kept) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) tot += (uint32_t)(start + j < N && key[j] >= T);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t g = start + j < N && key[j] > T, e = start + j < N && key[j] == T;
                        tot += g | e << 16;
                    }
                }
                const uint32_t incl = (uint32_t)wave_scan_incl((int)tot);
                before[st] = incl - tot;
                if (lane == 63) tots[st * 16 + wave] = incl;
            }
        }
        __syncthreads();
        // prefix over the (step, wave) totals: lane l holds entries 2l and 2l + 1
        const uint2 tv = lane < nsteps * 8 ? *(const uint2 *)&tots[2 * lane] : uint2{0u, 0u};
        const uint32_t pair_incl = (uint32_t)wave_scan_incl((int)(tv.x + tv.y));
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            if (st >= nsteps) break;
            const int e = st * 16 + wv;                // this wave's entry of the step (uniform)
            const uint32_t upto = (uint32_t)__builtin_amdgcn_readlane((int)pair_incl, e >> 1);   // through entry e | 1
            const uint32_t x1 = (uint32_t)__builtin_amdgcn_readlane((int)tv.y, e >> 1), x0 = (uint32_t)__builtin_amdgcn_readlane((int)tv.x, e >> 1);
            uint32_t excl = upto - x1 - ((e & 1) ? 0u : x0) + before[st];   // everything before this thread's 4 tokens
            const int start = st * kSelThreads * 4 + tid * 4;
            uint32_t key[4];
            load4(start, key);
            if (all_equal_kept) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool g = start + j < N && key[j] >= T;
                    if (g && (int)excl < k) row[excl] = start + j;   // (excl < k always holds; the test keeps a write in its row)
                    excl += (uint32_t)g;
                }
                continue;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool g = start + j < N && key[j] > T, eq = start + j < N && key[j] == T;
                const int g_before = (int)(excl & 0xFFFFu), e_before = (int)(excl >> 16);
                // a larger key goes behind the larger ones and the kept equal ones before it; an equal one is kept
                // while fewer than rem came before it, and then sits at that same place
                const int slot = g_before + min(e_before, rem);
                if ((g || (eq && e_before < rem)) && slot < k) row[slot] = start + j;   // (slot < k always holds; the test keeps a write in its row)
                excl += (uint32_t)g | (uint32_t)eq << 16;
            }
        }
        return;
    }
    int gt_run = 0, eq_run = 0, buf = 0;
    for (int base = 0; base < N; base += kSelThreads * 4, buf ^= 1) {
        // 4 consecutive tokens per thread: their flags are summed in the thread, one scan per wave, and the 16
        // wave totals (in token order) are read and scanned by every wave after the barrier
        const int start = base + tid * 4;
        uint32_t key[4];
        load4(start, key);
        int f[4], tot = 0;                             // packed counts: larger | equal << 16
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[j] = start + j < N ? (int)(key[j] > T) | ((int)(key[j] == T) << 16) : 0;
            tot += f[j];
        }
        const int incl = wave_scan_incl(tot);
        if (lane == 63) sub_tot[buf * 16 + wave] = incl;
        __syncthreads();
        const int tv = lane < 16 ? sub_tot[buf * 16 + lane] : 0;
        const int ti = wave_scan_incl(tv);
        const int run = __builtin_amdgcn_readlane(ti, 15);
        int excl = __builtin_amdgcn_readlane(ti, wv) - __builtin_amdgcn_readlane(tv, wv) + incl - tot;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int g_before = gt_run + (excl & 0xFFFF), e_before = eq_run + (excl >> 16);
            int slot = -1;
            if (f[j] & 1)
                slot = g_before + min(e_before, rem);
            else if (f[j] && e_before < rem)
                slot = g_before + e_before;
            if (slot >= 0 && slot < k) row[slot] = start + j;   // slot < k always holds; the test keeps a write in its row
            excl += f[j];
        }
        gt_run += run & 0xFFFF;
        eq_run += run >> 16;
    }
}

// ------------------------------------------------------------------------------------------------------
// The same selection with SEVERAL workgroups per unit (prompts of up to kChMaxChunks * 4096 tokens): launches
// over (unit, 4096-token chunk), no atomics in memory, no waiting between workgroups.  Every kernel requests
// all it reads from memory at its start (addresses clamped with launch parameters, validity applied when the
// values are used), so that a workgroup pays one memory round trip, not one per step.
//   sel_hist_kernel       streams the score rows once: summed-score keys to the workspace (several heads only)
//                         and, per chunk, a histogram of the keys' top 11 bits over the candidates.
//   sel_unit_hist_kernel  (more than kChDirect chunks per unit) adds a unit's chunk histograms up.
//   sel_cand_kernel       every workgroup takes its unit's histogram, finds the bin b1 the weakest kept heavy
//                         hitter falls into, counts its chunk's keys above that bin and copies those inside it
//                         (the "bin candidates") to the unit's list, behind those of the chunks before it.
//   sel_write_kernel      every workgroup settles the remaining 21 bits on the unit's bin candidates (two
//                         histogram passes over registers), counts what precedes its chunk, and compacts its
//                         chunk in order to the slots that follow.
// Workspace, in 32-bit words: keys [units][Lp] (several heads only; Lp = L rounded up to 4), bin candidates
// [units][nchunk*4096], chunk histograms [units][nchunk][1024] (two 16-bit counts per word), unit histograms
// [units][2048], per chunk four counts [units][nchunk][4] (bin candidates of the unit, keys above the bin in
// this chunk, the bin, bin candidates of the chunks before this one).
constexpr int kCh = 4096;              // tokens per chunk
constexpr int kChThreads = 256;        // 4 waves
constexpr int kChMaxChunks = 1024;     // most chunks of one unit
constexpr int kChDirect = 8;           // up to this many chunks sel_cand_kernel adds the chunk histograms itself
constexpr int kChCandRegs = 20;        // bin candidates per thread that sel_write_kernel holds in registers

struct SelWs {
    uint32_t *keys, *cand, *hist;
    int *uhist, *cnt;
    long Lp;
    int nchunk, units;
};

// Workgroup b of a launch over (unit, part), `parts` parts per unit: the hardware deals consecutive workgroups
// round-robin to the eight dies, each with an L2 of its own, so all parts of a unit are given numbers that are
// equal modulo 8 -- what one kernel writes for a unit is then still in the L2 of the die whose workgroups read
// it in the next (only speed depends on this).  Grids are sized by sel_grid_units(); false = no such unit.
__device__ __forceinline__ bool sel_map(unsigned b, int parts, int units, long &unit, int &part)
{
    if (units < 8) {                                       // fewer units than dies: spread every unit over all of them
        unit = b / (unsigned)parts;
        part = (int)(b % (unsigned)parts);
        return true;
    }
    const unsigned per = 8u * (unsigned)parts, g = b / per, r = b % per;
    unit = (long)g * 8 + (r & 7u);
    part = (int)(r >> 3);
    return unit < units;
}

static long sel_grid_units(long units) { return units < 8 ? units : (units + 7) / 8 * 8; }

__host__ __device__ inline long sel_ws_words(long units, int rep, long L)
{
    const long nchunk = (L + kCh - 1) / kCh, Lp = (L + 3) & ~3L;
    return units * ((rep > 1 ? Lp : 0) + nchunk * (kCh + kSelBins / 2 + 4) + kSelBins);
}

static SelWs sel_ws_carve(void *workspace, long units, int rep, long L)
{
    SelWs w;
    w.nchunk = (int)((L + kCh - 1) / kCh);
    w.units = (int)units;
    w.Lp = (L + 3) & ~3L;
    w.keys = (uint32_t *)workspace;
    w.cand = w.keys + (rep > 1 ? units * w.Lp : 0);
    w.hist = w.cand + units * (long)w.nchunk * kCh;
    w.uhist = (int *)(w.hist + units * (long)w.nchunk * (kSelBins / 2));
    w.cnt = w.uhist + units * (long)kSelBins;
    return w;
}

// Budgets of a unit: false when they are out of range.  N = candidates (tokens before the recent window).
__device__ __forceinline__ bool sel_budgets(long r, long h, long L, long idx_stride, int &N, int &k, int &rw)
{
    if (r < 0 || h < 0 || r > L || h > L - r || h + r > idx_stride) return false;
    N = (int)(L - r), k = (int)h, rw = (int)r;
    return true;
}

// Inclusive prefix sum over the 256 threads of a workgroup (tot[4] in LDS; one barrier); also the grand total.
__device__ __forceinline__ int block_scan_incl(int v, int *tot, int lane, int wv, int &total)
{
    int incl = wave_scan_incl(v);
    if (lane == 63) tot[wv] = incl;
    __syncthreads();
    const int t0 = tot[0], t1 = tot[1], t2 = tot[2], t3 = tot[3];
    incl += (wv > 0 ? t0 : 0) + (wv > 1 ? t1 : 0) + (wv > 2 ? t2 : 0);
    total = t0 + t1 + t2 + t3;
    return incl;
}

// Walk the 2048 bins c[.] (thread t holds bins 8t .. 8t+7) from the top: the bin in which the running count
// reaches `want` (1 <= want <= total) and how many of that bin are wanted.  The owning thread writes out[0..1]
// and returns the bin's place in its c[.]; the others return -1.
__device__ __forceinline__ int find_from_top(const int c[8], int want, int *tot, int *out, int tid, int lane, int wv)
{
    int mine = 0, total, own = -1;
#pragma unroll
    for (int j = 0; j < 8; ++j) mine += c[j];
    const int incl = block_scan_incl(mine, tot, lane, wv, total);
    int run = total - incl;                                // count in the bins above this thread's
#pragma unroll
    for (int j = 7; j >= 0; --j) {
        if (run < want && want <= run + c[j]) {
            out[0] = 8 * tid + j;
            out[1] = want - run;
            own = j;
        }
        run += c[j];
    }
    return own;
}

__device__ __forceinline__ void unpack_counts(const uint4 &v, int c[8])
{
    c[0] = v.x & 0xFFFF, c[1] = v.x >> 16, c[2] = v.y & 0xFFFF, c[3] = v.y >> 16;
    c[4] = v.z & 0xFFFF, c[5] = v.z >> 16, c[6] = v.w & 0xFFFF, c[7] = v.w >> 16;
}

template <int REP, bool FROM_FLOAT>
__global__ __launch_bounds__(kChThreads) void sel_hist_kernel(const float *__restrict__ A, SelWs w, int rep_rt, long L,
                                                              const int *__restrict__ n_hh,
                                                              const int *__restrict__ n_rw, long idx_stride)
{
    __shared__ int hist[kSelBins];
    const int rep = REP ? REP : rep_rt;
    long unit;
    int chunk;
    if (!sel_map(blockIdx.x, w.nchunk, w.units, unit, chunk)) return;
    const long base = (long)chunk * kCh;
    const int tid = threadIdx.x, lane = tid & 63;
    const long r_ = n_rw[unit], h_ = n_hh[unit];
    const float *rows = A + unit * rep * L;
    for (int b = tid; b < kSelBins; b += kChThreads) hist[b] = 0;
    int N = 0, k = 0, rw;
    bool live = false;
    for (int e0 = 0; e0 < 16; e0 += 4) {
        float s[4];
        if (REP) {
            float x[4][REP ? REP : 1];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long i = min(base + (e0 + e) * kChThreads + (long)tid, L - 1);   // clamped: no branch at the loads
#pragma unroll
                for (int h = 0; h < REP; ++h) x[e][h] = rows[h * L + i];
            }
            if (e0 == 0) {                                 // the first loads are on their way: now look at the budgets
                live = sel_budgets(r_, h_, L, idx_stride, N, k, rw) && k != 0 && k != N && base < N;
                __syncthreads();                           // (the cleared histogram)
                if (!live) return;                         // nothing is selected by score here / no candidate in this chunk
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s[e] = x[e][0];
#pragma unroll
                for (int h = 1; h < REP; ++h) s[e] = s[e] + x[e][h];                    // head order, one rounding per add
            }
        } else {
            if (e0 == 0) {
                live = sel_budgets(r_, h_, L, idx_stride, N, k, rw) && k != 0 && k != N && base < N;
                __syncthreads();
                if (!live) return;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long i = min(base + (e0 + e) * kChThreads + (long)tid, L - 1);
                s[e] = rows[i];
                for (int h = 1; h < rep; ++h) s[e] = s[e] + rows[h * L + i];
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long i = base + (e0 + e) * kChThreads + tid;
            const uint32_t key = score_key(s[e]);
            if (!FROM_FLOAT && i < N) w.keys[unit * w.Lp + i] = key;
            hist_add(hist, i < N, (int)(key >> 21), lane);
        }
    }
    __syncthreads();
    uint4 o;                                               // (a chunk holds 4096 tokens: a count fits 16 bits)
    o.x = (uint32_t)hist[8 * tid + 0] | ((uint32_t)hist[8 * tid + 1] << 16);
    o.y = (uint32_t)hist[8 * tid + 2] | ((uint32_t)hist[8 * tid + 3] << 16);
    o.z = (uint32_t)hist[8 * tid + 4] | ((uint32_t)hist[8 * tid + 5] << 16);
    o.w = (uint32_t)hist[8 * tid + 6] | ((uint32_t)hist[8 * tid + 7] << 16);
    reinterpret_cast<uint4 *>(w.hist + (unit * w.nchunk + chunk) * (long)(kSelBins / 2))[tid] = o;
}

// grid (units, 8): workgroup j of a unit adds bins 256j .. 256j+255 of the chunks that hold candidates
__global__ __launch_bounds__(kChThreads) void sel_unit_hist_kernel(SelWs w, long L, const int *__restrict__ n_hh,
                                                                   const int *__restrict__ n_rw, long idx_stride)
{
    long unit;
    int part;
    if (!sel_map(blockIdx.x, 8, w.units, unit, part)) return;
    const int bin = part * 256 + threadIdx.x;
    int N, k, rw;
    if (!sel_budgets(n_rw[unit], n_hh[unit], L, idx_stride, N, k, rw) || k == 0 || k == N) return;
    const int nc = (N + kCh - 1) / kCh;
    const uint16_t *hp = reinterpret_cast<const uint16_t *>(w.hist + unit * w.nchunk * (long)(kSelBins / 2)) + bin;
    int sum = 0;
    for (int q0 = 0; q0 < nc; q0 += 8) {
        int v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = hp[(long)min(q0 + j, nc - 1) * kSelBins];
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += q0 + j < nc ? v[j] : 0;
    }
    w.uhist[unit * kSelBins + bin] = sum;
}

template <bool FROM_FLOAT, bool DIRECT>
__global__ __launch_bounds__(kChThreads) void sel_cand_kernel(const float *__restrict__ A, SelWs w, long L,
                                                              const int *__restrict__ n_hh,
                                                              const int *__restrict__ n_rw, long idx_stride)
{
    __shared__ int tot[4], found[4], fill[2];
    long unit;
    int chunk;
    if (!sel_map(blockIdx.x, w.nchunk, w.units, unit, chunk)) return;
    const long base = (long)chunk * kCh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    // ---- everything this workgroup reads, requested at once
    const long r_ = n_rw[unit], h_ = n_hh[unit];
    uint32_t kk[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const long i = min(base + e * kChThreads + (long)tid, L - 1);
        kk[e] = FROM_FLOAT ? __float_as_uint(A[unit * L + i]) : w.keys[unit * w.Lp + i];
    }
    const uint32_t *hrow = w.hist + unit * w.nchunk * (long)(kSelBins / 2);
    uint4 hv[DIRECT ? kChDirect : 2];
    if (DIRECT) {
#pragma unroll
        for (int q = 0; q < kChDirect; ++q)
            hv[q] = reinterpret_cast<const uint4 *>(hrow + (long)min(q, w.nchunk - 1) * (kSelBins / 2))[tid];
    } else {
        hv[0] = reinterpret_cast<const uint4 *>(w.uhist + unit * kSelBins)[2 * tid];
        hv[1] = reinterpret_cast<const uint4 *>(w.uhist + unit * kSelBins)[2 * tid + 1];
    }
    if (tid < 2) fill[tid] = 0;
    int N, k, rw;
    if (!sel_budgets(r_, h_, L, idx_stride, N, k, rw)) return;
    if (k == 0 || k == N || base >= N) return;
    const int nc = (N + kCh - 1) / kCh;
    // ---- the unit's histogram and the bin b1 where the count from the top reaches k
    int c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (DIRECT) {
#pragma unroll
        for (int q = 0; q < kChDirect; ++q) {
            int cq[8];
            unpack_counts(hv[q], cq);
#pragma unroll
            for (int j = 0; j < 8; ++j) c[j] += q < nc ? cq[j] : 0;
        }
    } else {
        c[0] = hv[0].x, c[1] = hv[0].y, c[2] = hv[0].z, c[3] = hv[0].w;
        c[4] = hv[1].x, c[5] = hv[1].y, c[6] = hv[1].z, c[7] = hv[1].w;
    }
    const int own = find_from_top(c, k, tot, found, tid, lane, wv);
    // bin candidates of the unit (M) and of the chunks before this one
    if (DIRECT) {
        if (own >= 0) {
            int all = 0, before = 0;
#pragma unroll
            for (int q = 0; q < kChDirect; ++q) {
                int cq[8];
                unpack_counts(hv[q], cq);
                int x = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) x = own == j ? cq[j] : x;
                all += q < nc ? x : 0;
                before += q < chunk ? x : 0;
            }
            found[2] = all;
            found[3] = before;
        }
        __syncthreads();
    } else {
        __syncthreads();
        const uint16_t *hb = reinterpret_cast<const uint16_t *>(hrow) + found[0];
        int mine = 0, bef = 0;
#pragma unroll
        for (int j = 0; j < kChMaxChunks / kChThreads; ++j) {
            const int q = tid + j * kChThreads;
            const int x = q < nc ? (int)hb[(long)q * kSelBins] : 0;
            mine += x;
            bef += q < chunk ? x : 0;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            mine += __shfl_xor(mine, d, 64);
            bef += __shfl_xor(bef, d, 64);
        }
        if (tid < 2) found[2 + tid] = 0;
        __syncthreads();
        if (lane == 0) {
            atomicAdd(&found[2], mine);
            atomicAdd(&found[3], bef);
        }
        __syncthreads();
    }
    const uint32_t b1 = (uint32_t)found[0];
    const int M = found[2], m_before = found[3];
    uint32_t *seg = w.cand + unit * w.nchunk * (long)kCh + m_before;
    int above = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const bool in = base + e * kChThreads + tid < N;
        const uint32_t key = FROM_FLOAT ? score_key(__uint_as_float(kk[e])) : kk[e];
        const uint32_t d = key >> 21;
        above += (int)(in && d > b1);
        const bool is_c = in && d == b1;
        const unsigned long long m = __ballot(is_c);
        if (m) {                                            // the wave's bin candidates take consecutive places
            int at = 0;
            if (lane == 0) at = atomicAdd(&fill[0], (int)__popcll(m));
            at = __builtin_amdgcn_readfirstlane(at);
            if (is_c) seg[at + (int)__popcll(m & ((1ull << lane) - 1ull))] = key;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) above += __shfl_xor(above, d, 64);
    if (lane == 0) atomicAdd(&fill[1], above);
    __syncthreads();
    if (tid == 0) {
        int4 o;
        o.x = M, o.y = fill[1], o.z = (int)b1, o.w = m_before;
        reinterpret_cast<int4 *>(w.cnt)[unit * w.nchunk + chunk] = o;
    }
}

template <bool FROM_FLOAT>
__global__ __launch_bounds__(kChThreads, 4) void sel_write_kernel(const float *__restrict__ A, SelWs w, long L,
                                                               const int *__restrict__ n_hh,
                                                               const int *__restrict__ n_rw,
                                                               int *__restrict__ idx, long idx_stride,
                                                               int *__restrict__ n_tok)
{
    __shared__ int hist[kSelBins];
    __shared__ int tot[4], found[2], acc[4], sub_tot[2][4];
    long unit;
    int chunk;
    if (!sel_map(blockIdx.x, w.nchunk, w.units, unit, chunk)) return;
    const int base = chunk * kCh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    // ---- everything this workgroup reads, requested at once
    const long r_ = n_rw[unit], h_ = n_hh[unit];
    const int4 own = reinterpret_cast<const int4 *>(w.cnt)[unit * w.nchunk + chunk];
    int ab[kChMaxChunks / kChThreads];                     // keys above the bin, chunk tid + 256 j
#pragma unroll
    for (int j = 0; j < kChMaxChunks / kChThreads; ++j)
        ab[j] = w.cnt[(unit * w.nchunk + min(tid + j * kChThreads, w.nchunk - 1)) * 4 + 1];
    // this chunk's keys for the compaction: round r, thread t holds tokens base + r*1024 + 4t .. + 3
    uint32_t key[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const long i = min((long)base + r * 1024 + 4 * tid + j, L - 1);
            key[r][j] = FROM_FLOAT ? __float_as_uint(A[unit * L + i]) : w.keys[unit * w.Lp + i];
        }
    const uint32_t *cand = w.cand + unit * w.nchunk * (long)kCh;
    const int cap = w.nchunk * kCh;
    uint32_t cd[kChCandRegs];                              // the unit's first 6144 bin candidates (usually all)
#pragma unroll
    for (int e = 0; e < kChCandRegs; ++e) cd[e] = cand[min(tid + e * kChThreads, cap - 1)];
    if (tid < 4) acc[tid] = 0;

    int N, k, rw;
    if (!sel_budgets(r_, h_, L, idx_stride, N, k, rw)) {
        if (chunk == 0 && tid == 0) n_tok[unit] = 0;
        return;
    }
    int *row = idx + unit * idx_stride;
    const int end = (int)min((long)base + kCh, L);
    for (int i = max(base, N) + tid; i < end; i += kChThreads) row[k + (i - N)] = i;       // the recent window
    if (chunk == 0 && tid == 0) n_tok[unit] = k + rw;
    if (k == 0 || base >= N) return;
    if (k == N) {
        for (int i = base + tid; i < min(end, N); i += kChThreads) row[i] = i;
        return;
    }
    const int nc = (N + kCh - 1) / kCh;
    const int M = own.x, m_before = own.w;
    const uint32_t b1 = (uint32_t)own.z;
    int above_all, above_before;
    {
        int all = 0, bef = 0;
#pragma unroll
        for (int j = 0; j < kChMaxChunks / kChThreads; ++j) {
            const int q = tid + j * kChThreads;
            all += q < nc ? ab[j] : 0;
            bef += q < chunk ? ab[j] : 0;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            all += __shfl_xor(all, d, 64);
            bef += __shfl_xor(bef, d, 64);
        }
        __syncthreads();                                   // (acc cleared)
        if (lane == 0) {
            atomicAdd(&acc[0], all);
            atomicAdd(&acc[1], bef);
        }
        __syncthreads();
        above_all = acc[0], above_before = acc[1];
    }
    // f(key, before): every bin candidate of the unit once; before = it belongs to a chunk before this one
    auto for_each_cand = [&](auto f) {
#pragma unroll
        for (int e = 0; e < kChCandRegs; ++e) {
            const int i = tid + e * kChThreads;
            if (i < M) f(cd[e], i < m_before);
        }
        for (int i = tid + kChCandRegs * kChThreads; i < M; i += kChThreads) f(cand[i], i < m_before);
    };
    // the 21 bits below the bin's: 11, then 10
    int rem = k - above_all;
    uint32_t T = 0;
#pragma unroll 1
    for (int level = 0; level < 2; ++level) {
        const int lo = level ? 0 : 10;
        const uint32_t dm = level ? 0x3FFu : 0x7FFu;
        for (int b = tid; b < kSelBins; b += kChThreads) hist[b] = 0;
        __syncthreads();
        for_each_cand([&](uint32_t x, bool) {
            const bool match = level == 0 || ((x >> 10) & 0x7FFu) == (T >> 10);
            if (match) atomicAdd(&hist[(x >> lo) & dm], 1);
        });
        __syncthreads();
        int c[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = hist[8 * tid + j];
        find_from_top(c, rem, tot, found, tid, lane, wv);
        __syncthreads();
        T |= (uint32_t)found[0] << lo;
        rem = found[1];
        __syncthreads();
    }
    const uint32_t Tfull = (b1 << 21) | T;                 // key of the weakest kept heavy hitter; `rem` of its equals are kept
    // larger / equal keys among the bin candidates of the chunks before this one
    {
        int g = 0, e = 0;
        for_each_cand([&](uint32_t x, bool before) {
            g += (int)(before && x > Tfull);
            e += (int)(before && x == Tfull);
        });
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            g += __shfl_xor(g, d, 64);
            e += __shfl_xor(e, d, 64);
        }
        if (lane == 0) {
            atomicAdd(&acc[2], g);
            atomicAdd(&acc[3], e);
        }
    }
    __syncthreads();
    int gt_run = above_before + acc[2], eq_run = acc[3];
    // ---- ordered compaction of this chunk: four rounds of 1024 tokens, 4 consecutive tokens per thread
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int start = base + r * 1024 + 4 * tid;
        if (base + r * 1024 >= N) break;                   // (uniform)
        int f[4], sum = 0;                                 // packed counts: larger | equal << 16
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t x = FROM_FLOAT ? score_key(__uint_as_float(key[r][j])) : key[r][j];
            f[j] = start + j < N ? (int)(x > Tfull) | ((int)(x == Tfull) << 16) : 0;
            sum += f[j];
        }
        const int incl = wave_scan_incl(sum);
        if (lane == 63) sub_tot[r & 1][wv] = incl;
        __syncthreads();
        const int t0 = sub_tot[r & 1][0], t1 = sub_tot[r & 1][1], t2 = sub_tot[r & 1][2], t3 = sub_tot[r & 1][3];
        int excl = incl - sum + (wv > 0 ? t0 : 0) + (wv > 1 ? t1 : 0) + (wv > 2 ? t2 : 0);
        const int run = t0 + t1 + t2 + t3;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int g_before = gt_run + (excl & 0xFFFF), e_before = eq_run + (excl >> 16);
            int slot = -1;
            if (f[j] & 1)
                slot = g_before + min(e_before, rem);
            else if (f[j] && e_before < rem)
                slot = g_before + e_before;
            if (slot >= 0 && slot < k) row[slot] = start + j;   // slot < k always holds; the test keeps a write in its row
            excl += f[j];
        }
        gt_run += run & 0xFFFF;
        eq_run += run >> 16;
    }
}

static std::atomic<int> g_select_path{0};

bool set_select_path(int path)
{
    if (path < 0 || path > 2) return false;
    g_select_path.store(path);
    return true;
}

// Several workgroups per unit pay three to four dependent launches and read the keys three times; they win when
// one workgroup per unit would leave most of the chip idle.
static bool select_chunked(int32_t units, int64_t L)
{
    const long nchunk = (L + kCh - 1) / kCh;
    if (L <= 0 || nchunk > kChMaxChunks || ((long)units + 7) * nchunk > 0x7FFFFFFFL) return false;
    const int path = g_select_path.load();
    if (path) return path == 2;
    return nchunk > 8 && units <= 128;                  // (prompts whose keys one workgroup cannot hold in LDS; measured)
}

size_t select_workspace_bytes(int32_t units, int32_t rep, int64_t L)
{
    if (units <= 0 || rep < 1 || L <= 0) return 0;
    if ((L + kCh - 1) / kCh > kChMaxChunks)                 // one workgroup per unit: only the summed-score keys
        return rep > 1 ? (size_t)units * (size_t)L * sizeof(uint32_t) : 0;
    return (size_t)sel_ws_words(units, rep, L) * sizeof(uint32_t);
}

template <bool FROM_FLOAT>
static void launch_chunked_tail(const float *A, const SelWs &w, int32_t units, int64_t L, const int32_t *n_hh,
                                const int32_t *n_rw, int32_t *idx, int64_t idx_stride, int32_t *n_tok, hipStream_t st)
{
    const long units8 = sel_grid_units(units);
    const dim3 grid((unsigned)(units8 * w.nchunk));
    if (w.nchunk <= kChDirect) {
        hipLaunchKernelGGL((sel_cand_kernel<FROM_FLOAT, true>), grid, dim3(kChThreads), 0, st, A, w, (long)L, n_hh, n_rw,
                           (long)idx_stride);
    } else {
        hipLaunchKernelGGL(sel_unit_hist_kernel, dim3((unsigned)(units8 * 8)), dim3(kChThreads), 0, st, w, (long)L, n_hh,
                           n_rw, (long)idx_stride);
        hipLaunchKernelGGL((sel_cand_kernel<FROM_FLOAT, false>), grid, dim3(kChThreads), 0, st, A, w, (long)L, n_hh,
                           n_rw, (long)idx_stride);
    }
    hipLaunchKernelGGL((sel_write_kernel<FROM_FLOAT>), grid, dim3(kChThreads), 0, st, A, w, (long)L, n_hh, n_rw, idx,
                       (long)idx_stride, n_tok);
}

int launch_select(int32_t units, int32_t rep, int64_t L, const float *A, const int32_t *n_hh,
                  const int32_t *n_rw, int32_t *idx, int64_t idx_stride, int32_t *n_tok, void *workspace,
                  hipStream_t st)
{
    if (units == 0) return MINIKV_OK;
    if (select_chunked(units, L)) {
        const SelWs w = sel_ws_carve(workspace, units, rep, L);
        const dim3 grid((unsigned)(sel_grid_units(units) * w.nchunk));
        auto k1 = rep == 1   ? sel_hist_kernel<1, true>
                  : rep == 2 ? sel_hist_kernel<2, false>
                  : rep == 4 ? sel_hist_kernel<4, false>
                  : rep == 8 ? sel_hist_kernel<8, false>
                             : sel_hist_kernel<0, false>;
        hipLaunchKernelGGL(k1, grid, dim3(kChThreads), 0, st, A, w, rep, (long)L, n_hh, n_rw, (long)idx_stride);
        if (rep == 1)
            launch_chunked_tail<true>(A, w, units, L, n_hh, n_rw, idx, idx_stride, n_tok, st);
        else
            launch_chunked_tail<false>(A, w, units, L, n_hh, n_rw, idx, idx_stride, n_tok, st);
        return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
    }
    // keys stay in LDS when the whole prompt fits beside the fixed part
    int dev = 0, max_lds = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
        return MINIKV_ELAUNCH;
    long cap = ((long)max_lds - kSelFixedWords * 4) / 4;
    if (cap > kSelMaxCached) cap = kSelMaxCached;
    int cached = L > 0 && L <= cap;
    size_t lds = (size_t)kSelFixedWords * 4 + (cached ? (size_t)((L + 3) / 4 * 4) * 4 : 0);
    // with 2, 4 or 8 heads per unit and the keys held in LDS, the select kernel adds the heads' rows itself while
    // it reads them; otherwise (other head counts, or prompts whose keys are read again in every pass) the
    // streaming kernel leaves the summed-score keys in the workspace first
    const bool fused = cached && (rep == 2 || rep == 4 || rep == 8);
    auto kern = rep == 1            ? select_kernel<true, 1>
                : !fused            ? select_kernel<false, 1>
                : rep == 2          ? select_kernel<true, 2>
                : rep == 4          ? select_kernel<true, 4>
                                    : select_kernel<true, 8>;
    if (cached && lds > 48 * 1024 &&
        hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        cached = 0;                                    // read the keys from memory in every pass instead
        lds = (size_t)kSelFixedWords * 4;
        if (rep > 1) kern = select_kernel<false, 1>;
    }
    uint32_t *keys = (uint32_t *)workspace;
    if (rep > 1 && L > 0 && kern == select_kernel<false, 1>) {
        const int nchunk = (int)((L + 4095) / 4096);
        auto k1 = rep == 2 ? score_key_kernel<2> : rep == 4 ? score_key_kernel<4> : rep == 8 ? score_key_kernel<8>
                                                                                            : score_key_kernel<0>;
        hipLaunchKernelGGL(k1, dim3((unsigned)((long)units * nchunk)), dim3(256), 0, st, A, keys, rep, (long)L,
                           nchunk);
        if (hipGetLastError() != hipSuccess) return MINIKV_ELAUNCH;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)units), dim3(kSelThreads), lds, st, A, keys, (long)L, n_hh, n_rw,
                       idx, (long)idx_stride, n_tok, cached);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

}  // namespace minikv
