// Prefill attention that also returns the cumulative attention score of every prompt token, in memory linear
// in the prompt length (Section 3.2; Algorithm 1 line 2): X_O = softmax(sm_scale Q K^T) V on the causal part,
// LSE per query row, A_cumul = column sums of the softmax matrix.
//
// Two kernels, as in Section 3.2, re-tiled for 64-lane waves and the 32x32x16 fp16 matrix instruction:
//   prefill_fwd_kernel     row blocks in parallel.  A workgroup of 4 waves owns 128 queries (32 per wave) and
//                          walks the keys in tiles of 64 through LDS.  Scores are computed TRANSPOSED,
//                          S^T = K Q^T, so that a lane holds one query column: the running max / sum of the
//                          online softmax are per-lane scalars (one exchange between the two half-waves per
//                          tile), the rescale of the output is a per-lane multiply, and the fp32 scores, once
//                          turned into fp16 weights, ARE the B operand of O^T = V^T P^T without any shuffle
//                          (the key order inside a 16-key step is whatever the accumulator layout gives; the
//                          V^T operand is read in the same order).  V^T tiles come from a transposed copy of V
//                          that prefill_vt_kernel writes once into the workspace: transposing inside the key
//                          loop (2-byte LDS stores) cost as much as the rest of the loop together.
//   prefill_colsum_kernel  column blocks in parallel.  A workgroup owns 128 keys (32 per wave, their K rows
//                          held in registers as the B operand), walks the queries from the diagonal down in
//                          tiles of 64 through LDS, recomputes S = Q K^T, normalises with the saved LSE and
//                          adds the weights of its key column in the lane: no atomics, one exchange at the end.
#include "common.h"

#include <type_traits>

namespace minikv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kPfD = 128;            // head dimension
constexpr int kPfM = 128;            // queries per workgroup (forward) / keys per workgroup (column sums)
constexpr int kPfN = 64;             // keys (forward) / queries (column sums) per LDS tile
constexpr int kPfKRow = kPfD + 8;    // halves per row of a row-major tile in LDS (16-byte pad)
constexpr int kPfVRow = kPfN + 4;    // halves per row of the transposed V tile in LDS: 34 words, so that the 64-bit
                                     // fragment reads of 32 consecutive rows fall on 32 different bank pairs
constexpr int kPfKTile = kPfN * kPfKRow;   // halves of one row-major tile in LDS
constexpr int kPfVTile = kPfD * kPfVRow;   // halves of one transposed V tile in LDS
constexpr size_t kPfFwdLds = (size_t)2 * (kPfKTile + kPfVTile) * sizeof(_Float16);
constexpr int kWaitVm0 = 0x0F70;      // s_waitcnt vmcnt(0), other counters untouched
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct PrefillArgs {
    const _Float16 *Q, *K, *V;
    _Float16 *Vt;                    // workspace: V transposed, [B*Hkv][128][Lp], zero beyond L
    long Lp;                         // L rounded up to a multiple of 64
    _Float16 *XO;
    float *lse, *A_cumul;
    int Hq, rep, nblk;
    long L;
    float scale_log2;                // sm_scale * log2(e): the softmax runs on powers of two
};

__device__ __forceinline__ float16v mfma32(half8 a, half8 b, float16v c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// Row of accumulator element i (0..15) inside a 32x32 result tile, for a lane of half-wave g.
__device__ __forceinline__ int acc_row(int i, int g) { return (i >> 2) * 8 + g * 4 + (i & 3); }

// Tiles come from global memory through buffer loads: a descriptor (base, byte size) per head in scalar
// registers, ONE loop-invariant byte offset per lane and a scalar offset per tile and chunk, so the loop spends
// no vector instructions on addresses; bytes beyond the size read as zero (rows past the end of the prompt).
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
constexpr int kRawBufferFlags = 0x00020000;   // raw buffer, 32-bit data format
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, kRawBufferFlags);
}
struct TileRegs {
    uint4 c[4];
};
// One tile of 64 rows x 128 halves (rows are 256 bytes, so chunk k of the tile is at byte 16 k): 4 chunks of 16
// bytes per thread, coalesced.  lane_off = 16 * tid.
__device__ __forceinline__ TileRegs load_tile(__amdgpu_buffer_rsrc_t rs, unsigned lane_off, unsigned tile_off)
{
    TileRegs t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, tile_off + 4096u * i, 0);
        t.c[i] = make_uint4(v[0], v[1], v[2], v[3]);
    }
    return t;
}
__device__ __forceinline__ void store_tile_rowmajor(_Float16 *lds, const TileRegs &t, int tid)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int chunk = tid + 256 * i;
        *(uint4 *)(lds + (chunk >> 4) * kPfKRow + (chunk & 15) * 8) = t.c[i];
    }
}
// One tile of 128 channels x 64 keys of the transposed V: chunk = 8 keys of one channel, channel = chunk / 8.
// lane_off = (tid / 8) * row_bytes + (tid % 8) * 16; chunk tid + 256 i is 32 i rows further down.
__device__ __forceinline__ TileRegs load_tile_vt(__amdgpu_buffer_rsrc_t rs, unsigned lane_off, unsigned key_off,
                                                 unsigned row_bytes)
{
    TileRegs t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, key_off + 32u * i * row_bytes, 0);
        t.c[i] = make_uint4(v[0], v[1], v[2], v[3]);
    }
    return t;
}
__device__ __forceinline__ void store_tile_vt(_Float16 *lds, const TileRegs &t, int tid)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int chunk = tid + 256 * i;
        uint2 *p = (uint2 *)(lds + (chunk >> 3) * kPfVRow + (chunk & 7) * 8);       // rows are 8-byte aligned only
        p[0] = make_uint2(t.c[i].x, t.c[i].y);
        p[1] = make_uint2(t.c[i].z, t.c[i].w);
    }
}

// V [heads][L][128] -> Vt [heads][128][Lp], keys L .. Lp-1 zero (they meet zero weights, which must not meet NaN).
__global__ __launch_bounds__(256) void prefill_vt_kernel(const _Float16 *__restrict__ V, _Float16 *__restrict__ Vt,
                                                         long L, long Lp)
{
    __shared__ __align__(16) _Float16 tile[kPfN * kPfKRow];
    const int tid = threadIdx.x;
    const long head = blockIdx.y, key0 = (long)blockIdx.x * kPfN;
    const _Float16 *vh = V + head * L * kPfD;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int chunk = tid + 256 * i;
        const long row = key0 + (chunk >> 4);
        uint4 c = {0u, 0u, 0u, 0u};
        if (row < L) c = *(const uint4 *)(vh + row * kPfD + (chunk & 15) * 8);
        *(uint4 *)(tile + (chunk >> 4) * kPfKRow + (chunk & 15) * 8) = c;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int chunk = tid + 256 * i;
        const int d = chunk >> 3, kc = (chunk & 7) * 8;
        half8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = tile[(kc + j) * kPfKRow + d];
        *(half8 *)(Vt + (head * kPfD + d) * Lp + key0 + kc) = v;
    }
}

__global__ __launch_bounds__(256, 2) void prefill_fwd_kernel(PrefillArgs a)
{
    extern __shared__ __align__(16) _Float16 pf_lds[];
    _Float16 *Ks = pf_lds, *Vt = pf_lds + 2 * kPfKTile;     // [2][64][136] and [2][128][68] halves

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, g = lane >> 5;
    // heaviest row blocks (the last ones: they see the most keys) first
    const int nbh = gridDim.x / a.nblk;
    const int qb = a.nblk - 1 - (int)(blockIdx.x / nbh);
    const long bh = blockIdx.x % nbh;
    const long kvh = (bh / a.Hq) * (a.Hq / a.rep) + (bh % a.Hq) / a.rep;
    const long L = a.L;
    const _Float16 *Qh = a.Q + bh * L * kPfD, *Kh = a.K + kvh * L * kPfD, *Vth = a.Vt + kvh * kPfD * a.Lp;

    const long q0 = (long)qb * kPfM + wave * 32;       // first query of this wave
    const long query = q0 + r;                         // this lane's query column
    const long qrow = query < L ? query : L - 1;
    half8 qf[8];                                       // B operand of S^T = K Q^T: Q[query][16 ks + 8 g ..]
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const half8 *)(Qh + qrow * kPfD + ks * 16 + g * 8);

    float16v o[4];                                     // O^T: o[db][i] = out[query][32 db + acc_row(i, g)]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.0f;
    float m = -INFINITY, l = 0.0f;                     // running max (shared by both half-waves), this lane's part of the sum

    const long kend = min((long)(qb + 1) * kPfM, L);   // keys 0 .. kend-1 are visible to some query of the block
    const int ntiles = (int)((kend + kPfN - 1) / kPfN);
    const float c = a.scale_log2;                      // > 0: the running max is kept on the raw scores
    // Two LDS buffers, one barrier per tile.  The global loads of tile n+1 are issued after the score products
    // of tile n (whose K fragments can then use those registers) and stored to the other buffer at the end of
    // the iteration, behind the softmax and the output products.
    const __amdgpu_buffer_rsrc_t krs = buffer_of(Kh, (unsigned)(L * kPfD * 2)), vrs = buffer_of(Vth, (unsigned)(kPfD * a.Lp * 2));
    const unsigned row_bytes = (unsigned)(a.Lp * 2), k_lane = tid * 16u, v_lane = (tid >> 3) * row_bytes + (tid & 7) * 16u;
    constexpr unsigned kKTileBytes = kPfN * kPfD * 2, kVTileBytes = kPfN * 2;
    TileRegs kr = load_tile(krs, k_lane, 0), vr = load_tile_vt(vrs, v_lane, 0, row_bytes);
    store_tile_rowmajor(Ks, kr, tid);
    store_tile_vt(Vt, vr, tid);
    // Every load so far (the Q rows among them) has returned by now, since loads return in order and the stores
    // above needed the last ones.  Saying so keeps the compiler from guarding the Q registers inside the loop
    // with counts that would also wait for the prefetch.
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __syncthreads();
    for (int n = 0; n < ntiles; ++n) {
        const _Float16 *Kc = Ks + (n & 1) * kPfKTile, *Vc = Vt + (n & 1) * kPfVTile;
        const long key0 = (long)n * kPfN;
        if (key0 <= q0 + 31) {                         // else no query of this wave sees the tile (uniform in the wave)
            // all 8 K fragments of the first 32 keys are requested before the first product; each is replaced
            // by the fragment of the second 32 keys as soon as it is consumed
            float16v s[2];
            half8 kf[8];
            const _Float16 *kp = Kc + r * kPfKRow + g * 8;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) kf[ks] = *(const half8 *)(kp + ks * 16);
#pragma unroll
            for (int i = 0; i < 16; ++i) s[0][i] = 0.0f, s[1][i] = 0.0f;
            __builtin_amdgcn_sched_barrier(0);         // keep the requests above the products (the scheduler would
                                                       // otherwise pull each one down to its use to save registers)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                s[0] = mfma32(kf[ks], qf[ks], s[0]);
                kf[ks] = *(const half8 *)(kp + 32 * kPfKRow + ks * 16);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) s[1] = mfma32(kf[ks], qf[ks], s[1]);
            if (n + 1 < ntiles) {
                kr = load_tile(krs, k_lane, (n + 1) * kKTileBytes);
                vr = load_tile_vt(vrs, v_lane, (n + 1) * kVTileBytes, row_bytes);
            }
            float mx = m;
            if (key0 + kPfN - 1 > q0) {                // the diagonal crosses the tile: keys after the query are masked
                const int rel = (int)(query - key0);   // keys at tile offsets 0 .. rel are visible to this lane
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        if (t * 32 + acc_row(i, g) > rel) s[t][i] = -INFINITY;
                        mx = fmaxf(mx, s[t][i]);
                    }
            } else {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[t][i]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));    // the other half-wave holds the other 32 keys of the column
            const float alpha = __builtin_amdgcn_exp2f((m - mx) * c);   // m = -inf at the first tile: alpha = 0
            m = mx;
            const float mc = -mx * c;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
            }
            // Output products in four steps of 16 keys (step q: keys 32 (q>>1) + 16 (q&1) + 4 g + {0..3} and the
            // same + 8, the accumulator's own order).  The V^T fragments of step q+1 are requested and the
            // weights of step q+1 computed while the four products of step q run.
            float psum = 0.0f;
            auto weights = [&](int q) -> half8 {           // B operand of step q: exp2 of its eight scores
                half8 pb;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[q >> 1][(q & 1) * 8 + j], c, mc));
                    psum += p;
                    pb[j] = (_Float16)p;
                }
                return pb;
            };
            const _Float16 *vbase = Vc + r * kPfVRow + g * 4;
            auto vfrag = [&](int q, int db) -> half8 {
                const _Float16 *vp = vbase + db * 32 * kPfVRow + q * 16;
                const half4 lo = *(const half4 *)vp, hi = *(const half4 *)(vp + 8);
                return half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            };
            half8 vf[4], vn[4], pb = weights(0), pn;
#pragma unroll
            for (int db = 0; db < 4; ++db) vf[db] = vfrag(0, db);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (q < 3) {
#pragma unroll
                    for (int db = 0; db < 4; ++db) vn[db] = vfrag(q + 1, db);
                }
                __builtin_amdgcn_sched_barrier(0);         // (the requests stay above the products)
                if (q < 3) pn = weights(q + 1);
#pragma unroll
                for (int db = 0; db < 4; ++db) o[db] = mfma32(vf[db], pb, o[db]);
                __builtin_amdgcn_sched_barrier(0);
                if (q < 3) {
                    pb = pn;
#pragma unroll
                    for (int db = 0; db < 4; ++db) vf[db] = vn[db];
                }
            }
            l = l * alpha + psum;
        } else if (n + 1 < ntiles) {                   // a wave that skips the tile still moves its share of the next one
            kr = load_tile(krs, k_lane, (n + 1) * kKTileBytes);
            vr = load_tile_vt(vrs, v_lane, (n + 1) * kVTileBytes, row_bytes);
        }
        if (n + 1 < ntiles) {                          // the other buffer was last read before the previous barrier
            store_tile_rowmajor(Ks + ((n + 1) & 1) * kPfKTile, kr, tid);
            store_tile_vt(Vt + ((n + 1) & 1) * kPfVTile, vr, tid);
        }
        __syncthreads();                               // tile n+1 is in place, everyone is done with tile n
    }

    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
    if (query < L) {
        if (g == 0) a.lse[bh * L + query] = (m * c + log2f(l)) * kLn2;
        _Float16 *orow = a.XO + (bh * L + query) * kPfD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int iq = 0; iq < 4; ++iq) {
                half4 h;
#pragma unroll
                for (int j = 0; j < 4; ++j) h[j] = (_Float16)(o[db][iq * 4 + j] * inv);
                *(half4 *)(orow + db * 32 + iq * 8 + g * 4) = h;
            }
    }
}

__global__ __launch_bounds__(256, 2) void prefill_colsum_kernel(PrefillArgs a)
{
    __shared__ __align__(16) _Float16 Qs[2 * kPfKTile];
    __shared__ __align__(16) float lse2[2 * kPfN];     // LSE of the tile's queries, in powers of two (two buffers each)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, g = lane >> 5;
    // column blocks in natural order: block 0 is seen by every query and is the heaviest
    const int nbh = gridDim.x / a.nblk;
    const int kb = (int)(blockIdx.x / nbh);
    const long bh = blockIdx.x % nbh;
    const long kvh = (bh / a.Hq) * (a.Hq / a.rep) + (bh % a.Hq) / a.rep;
    const long L = a.L;
    const _Float16 *Qh = a.Q + bh * L * kPfD, *Kh = a.K + kvh * L * kPfD;
    const float *lseh = a.lse + bh * L;

    const long k0 = (long)kb * kPfM + wave * 32;       // first key of this wave
    const long key = k0 + r;                           // this lane's key column
    const long krow = key < L ? key : L - 1;
    half8 kf[8];                                       // B operand of S = Q K^T: K[key][16 ks + 8 g ..]
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = *(const half8 *)(Kh + krow * kPfD + ks * 16 + g * 8);

    float colsum = 0.0f;
    const float c = a.scale_log2;
    const int tile0 = (int)(((long)kb * kPfM) / kPfN), ntiles = (int)((L + kPfN - 1) / kPfN);
    const __amdgpu_buffer_rsrc_t qrs = buffer_of(Qh, (unsigned)(L * kPfD * 2));
    const unsigned q_lane = tid * 16u;
    constexpr unsigned kQTileBytes = kPfN * kPfD * 2;
    TileRegs qr = load_tile(qrs, q_lane, tile0 * kQTileBytes);
    float lr = 0.0f;
    if (tid < kPfN) lr = lseh[min((long)tile0 * kPfN + tid, L - 1)];
    store_tile_rowmajor(Qs, qr, tid);
    if (tid < kPfN) lse2[tid] = lr * kLog2e;
    __builtin_amdgcn_s_waitcnt(kWaitVm0);              // as in the first pass: the K rows have arrived
    if (tile0 + 1 < ntiles) {
        qr = load_tile(qrs, q_lane, (tile0 + 1) * kQTileBytes);
        if (tid < kPfN) lr = lseh[min((long)(tile0 + 1) * kPfN + tid, L - 1)];
    }
    __syncthreads();
    for (int n = tile0; n < ntiles; ++n) {
        const int cur = (n - tile0) & 1;
        const _Float16 *Qc = Qs + cur * kPfKTile;
        const float *lc = lse2 + cur * kPfN;
        if (n + 1 < ntiles) {
            store_tile_rowmajor(Qs + (cur ^ 1) * kPfKTile, qr, tid);
            if (tid < kPfN) lse2[(cur ^ 1) * kPfN + tid] = lr * kLog2e;
        }
        if (n + 2 < ntiles) {
            qr = load_tile(qrs, q_lane, (n + 2) * kQTileBytes);
            if (tid < kPfN) lr = lseh[min((long)(n + 2) * kPfN + tid, L - 1)];
        }
        const long qt0 = (long)n * kPfN;
        if (qt0 + kPfN - 1 >= k0) {                    // else every query of the tile precedes every key of this wave
            const bool edge = qt0 < k0 + 31 || qt0 + kPfN > L;   // the diagonal or the end of the prompt crosses the tile
            const int lo_q = (int)(key - qt0), hi_q = (int)min(L - qt0, (long)kPfN);   // tile rows lo_q .. hi_q-1 count
            // two copies of the tile's work, chosen per tile: only the few edge tiles pay for the masking
            auto tile = [&](auto masked) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    float16v s;
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[i] = 0.0f;
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        const half8 qf = *(const half8 *)(Qc + (t * 32 + r) * kPfKRow + ks * 16 + g * 8);
                        s = mfma32(qf, kf[ks], s);
                    }
#pragma unroll
                    for (int iq = 0; iq < 4; ++iq) {
                        const float4 ls = *(const float4 *)&lc[t * 32 + iq * 8 + g * 4];
                        const float lsv[4] = {ls.x, ls.y, ls.z, ls.w};
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[iq * 4 + j], c, -lsv[j]));
                            if (decltype(masked)::value) {
                                const int row = t * 32 + iq * 8 + g * 4 + j;
                                if (row < lo_q || row >= hi_q) p = 0.0f;
                            }
                            colsum += p;
                        }
                    }
                }
            };
            if (edge)
                tile(std::true_type{});
            else
                tile(std::false_type{});
        }
        __syncthreads();
    }
    colsum += __shfl_xor(colsum, 32, 64);
    if (g == 0 && key < L) a.A_cumul[bh * L + key] = colsum;
}

int launch_prefill(int32_t B, int32_t Hq, int32_t Hkv, int64_t L, const minikv_f16 *Q, const minikv_f16 *K,
                   const minikv_f16 *V, float sm_scale, minikv_f16 *XO, float *lse, float *A_cumul,
                   void *workspace, hipStream_t st)
{
    PrefillArgs a;
    a.Lp = (L + kPfN - 1) / kPfN * kPfN;
    a.Vt = (_Float16 *)workspace;
    a.Q = (const _Float16 *)Q, a.K = (const _Float16 *)K, a.V = (const _Float16 *)V;
    a.XO = (_Float16 *)XO, a.lse = lse, a.A_cumul = A_cumul;
    a.Hq = Hq, a.rep = Hq / Hkv, a.L = L, a.scale_log2 = sm_scale * kLog2e;
    a.nblk = (int)((L + kPfM - 1) / kPfM);
    const long blocks = (long)B * Hq * a.nblk;
    hipLaunchKernelGGL(prefill_vt_kernel, dim3((unsigned)(a.Lp / kPfN), (unsigned)(B * Hkv)), dim3(256), 0, st, a.V,
                       a.Vt, (long)L, a.Lp);
    if (hipGetLastError() != hipSuccess) return MINIKV_ELAUNCH;
    if (hipFuncSetAttribute((const void *)prefill_fwd_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kPfFwdLds) != hipSuccess)
        return MINIKV_ELAUNCH;
    hipLaunchKernelGGL(prefill_fwd_kernel, dim3((unsigned)blocks), dim3(256), kPfFwdLds, st, a);
    if (hipGetLastError() != hipSuccess) return MINIKV_ELAUNCH;
    if (A_cumul) {
        hipLaunchKernelGGL(prefill_colsum_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return MINIKV_ELAUNCH;
    }
    return MINIKV_OK;
}

}  // namespace minikv
