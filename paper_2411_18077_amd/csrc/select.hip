// Token selection at the end of the prefill (Section 3.1.2, Algorithm 1 line 3): per unit keep the recent
// window and, of the other prompt tokens, the n_hh with the largest cumulative attention score; write the
// kept positions in ascending order.
//
// Two kernels.
//   score_key_kernel   (only when a unit has several query heads) streams the rep fp32 score rows of a
//                      unit once, adds them in head order in fp32 and stores an order-preserving 32-bit
//                      key per token.  Grid over (unit, 4096-token chunk): the whole chip streams.
//   select_kernel      one workgroup of 16 waves per unit.  A radix select (11-bit digits of key - min key,
//                      from the top bit of the keys' range down; LDS histogram, scan from the top bin
//                      down) finds the key T of the weakest kept heavy hitter and how many tokens equal
//                      to T are kept; then one ordered compaction
//                      pass writes position i if key_i > T, or key_i == T and fewer than that many equal
//                      keys precede it, to slot (#larger before i) + min(#equal before i, kept equals).
//                      Equal scores therefore go to the earlier position and the output is ascending
//                      without a sort.  When the prompt fits, the keys are read from memory once and held
//                      in LDS (up to 32768 tokens = 128 KB) for the other passes.
#include "common.h"

namespace minikv {

constexpr int kSelThreads = 1024;      // 16 waves: one workgroup per unit
constexpr int kSelBins = 2048;         // 11-bit digits
constexpr int kSelLoads = 8;           // keys per thread in flight in a histogram pass
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

template <bool FROM_FLOAT>
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
    int *found = scan_tot + 16;                      // [2] digit, kept count below it
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
    const float *arow = A + u * L;
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

    // ---- the range [kmin, kmax] of the candidates' keys; the keys go to LDS on the way when they fit
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    for (int base = 0; base < N; base += kSelThreads * kSelRangeLoads) {
        uint32_t kk[kSelRangeLoads];
        // every load of the step is issued before the first is used: indices clamped, no branches
#pragma unroll
        for (int e = 0; e < kSelRangeLoads; ++e) kk[e] = gload(min(base + e * kSelThreads + tid, N - 1));
#pragma unroll
        for (int e = 0; e < kSelRangeLoads; ++e) {
            const int i = base + e * kSelThreads + tid;
            kk[e] = gkey(kk[e]);
            kmin = min(kmin, kk[e]);
            kmax = max(kmax, kk[e]);
            if (cached && i < N) ck[i] = kk[e];
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d, 64));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d, 64));
    }
    if (lane == 0) {
        scan_tot[wave] = (int)kmin;
        sub_tot[wave] = (int)kmax;
    }
    __syncthreads();
    for (int w = 0; w < 16; ++w) {
        kmin = min(kmin, (uint32_t)scan_tot[w]);
        kmax = max(kmax, (uint32_t)sub_tot[w]);
    }
    __syncthreads();

    // ---- radix select on x = key - kmin, 11 bits at a time from the top bit of kmax - kmin down (digits of
    // the RANGE, so that scores crowded into a few binades still spread over the histogram).  Bits hi and
    // above of T - kmin are known (`prefix`); `rem` = how many tokens sharing them are still to be kept.
    uint32_t prefix = 0;
    int rem = k;
    int hi = 32 - __clz((int)(kmax - kmin));          // 0 when all candidates are equal: T = kmin at once
    while (hi > 0) {
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
            bool match[kSelLoads], any = false;
#pragma unroll
            for (int e = 0; e < kSelLoads; ++e) {
                kk[e] -= kmin;
                match[e] = tok(e) < N && (hi == 32 || (kk[e] >> hi) == (prefix >> hi));
                any |= match[e];
            }
            if (__ballot(any) == 0) continue;          // after the first digit few tokens still share the prefix
#pragma unroll
            for (int e = 0; e < kSelLoads; ++e) hist_add(hist, match[e], (int)((kk[e] >> lo) & dm), lane);
        }
        __syncthreads();
        // bins from the top down, two per thread; the thread whose pair crosses `rem` owns the digit
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
        }
        __syncthreads();
        prefix |= (uint32_t)found[0] << lo;
        rem = found[1];
        hi = lo;
        __syncthreads();
    }

    // ---- ordered compaction
    const uint32_t T = kmin + prefix;
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

int launch_select(int32_t units, int32_t rep, int64_t L, const float *A, const int32_t *n_hh,
                  const int32_t *n_rw, int32_t *idx, int64_t idx_stride, int32_t *n_tok, void *workspace,
                  hipStream_t st)
{
    if (units == 0) return MINIKV_OK;
    uint32_t *keys = (uint32_t *)workspace;
    if (rep > 1 && L > 0) {
        const int nchunk = (int)((L + 4095) / 4096);
        auto k1 = rep == 2 ? score_key_kernel<2> : rep == 4 ? score_key_kernel<4> : rep == 8 ? score_key_kernel<8>
                                                                                            : score_key_kernel<0>;
        hipLaunchKernelGGL(k1, dim3((unsigned)((long)units * nchunk)), dim3(256), 0, st, A, keys, rep, (long)L,
                           nchunk);
        if (hipGetLastError() != hipSuccess) return MINIKV_ELAUNCH;
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
    auto kern = rep > 1 ? select_kernel<false> : select_kernel<true>;
    if (cached && lds > 48 * 1024 &&
        hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        cached = 0;                                    // read the keys from memory in every pass instead
        lds = (size_t)kSelFixedWords * 4;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)units), dim3(kSelThreads), lds, st, A, keys, (long)L, n_hh, n_rw,
                       idx, (long)idx_stride, n_tok, cached);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

}  // namespace minikv
