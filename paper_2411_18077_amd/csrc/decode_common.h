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
    float *ws;                   // split-K partials [B*Hq][nchunk+1][kPartialStride]
    float c1;                    // sm_scale * log2(e): scores are kept in the base-2 domain
    int Hq, Hkv, rep, Tcap, Rcap, chunk, nchunk;
};

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
