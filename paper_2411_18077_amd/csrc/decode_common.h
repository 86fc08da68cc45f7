// Declarations shared by the decode-attention translation units.
#pragma once

#include "common.h"

namespace minikv {

struct DecArgs {
    const uint16_t *q;           // [B][Hq][D] fp16
    const uint32_t *Kc, *Vc;
    const uint16_t *Ks, *Kz, *Vs, *Vz, *Rk, *Rv;
    const int32_t *q_len, *r_len;
    uint16_t *out;               // [B][Hq][D] fp16
    float *ws;                   // split-K partials (layout depends on the variant)
    int *cnt;                    // per-unit ticket counters of the single-launch kernel (zero between calls)
    int *cnt1;                   // ticket counters of the sub-groups, indexed by the sub-group's first slot
    int *redo;                   // counts (wave, unit) pairs redone with range-normalised operands (diagnostics)
    int first_slot;              // workgroups that fill the first wave slot of every SIMD
    int skew16;                  // sixteenths of a wave pair's range that its first wave takes
    float c1;                    // sm_scale * log2(e): scores are kept in the base-2 domain
    int Hq, Hkv, rep, Tcap, Rcap, chunk, nchunk;
    int units, hsets;            // B*Hkv; sets of 4 query heads per KV head (1 or 2)
    int hs_shift;                // log2(hsets)
    uint32_t hkv_magic, hkv_shift;   // exact division by Hkv: see fast_div()
    // the fused step (append + attend in one launch; all null / 0 otherwise): the new token's rows [B*Hkv][D]
    // (filed in Rk, Rv, which the step may write) and where the lengths after the append go
    const uint16_t *k_new, *v_new;
    int32_t *r_len_out;
    int append;
};

// n / d for any 32-bit n, with (magic, shift) from fast_div_setup(d) -- no integer divide on the device.
__host__ __device__ inline uint32_t fast_div(uint32_t n, uint32_t magic, uint32_t shift)
{
    const uint32_t hi = (uint32_t)(((uint64_t)n * magic) >> 32);
    return (uint32_t)(((uint64_t)hi + n) >> shift);
}
inline void fast_div_setup(uint32_t d, uint32_t &magic, uint32_t &shift)
{
    shift = 0;
    while ((1ull << shift) < d) shift++;
    magic = (uint32_t)((((1ull << shift) - d) << 32) / d + 1);
}

// Partial of (query row bq, chunk ch): [0] running max (base-2 domain), [1] sum of weights,
// [4..131] un-normalised output.  Chunk index nchunk is the fp16 residual.
__device__ inline float *partial_ptr(const DecArgs &a, int bq, int ch)
{
    return a.ws + ((size_t)bq * (a.nchunk + 1) + ch) * kPartialStride;
}

__device__ inline int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

int launch_decode_scalar(const DecArgs &a, int G, int units, hipStream_t st);
int launch_decode_tiled(const DecArgs &a, int G, int units, int variant, hipStream_t st);
int launch_merge(const DecArgs &a, int nq, hipStream_t st);

}  // namespace minikv
