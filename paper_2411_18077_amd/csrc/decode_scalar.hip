// Cross-check decode kernel: plain per-token loops in fp32, no tiling tricks.  It follows
// Algorithm 1 lines 17-19 of the MiniKV paper literally (scores of the dequantized keys and of the fp16
// residual keys, one softmax, weighted sum of dequantized and residual values) with a block-level
// online softmax, and exists so that the tuned kernels can be compared against a second GPU
// implementation that shares none of their indexing.  Also holds the split-K merge kernel and the
// variant dispatch.
#include "decode_common.h"

#include <hip/hip_fp16.h>

namespace minikv {

__device__ inline float hf(uint16_t h) { return __half2float(__ushort_as_half(h)); }

__device__ inline float wave_max(float v)
{
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float wave_sum(float v)
{
    for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int G>
__global__ __launch_bounds__(256) void decode_scalar_kernel(DecArgs a)
{
    constexpr int NCG = kD / G;
    constexpr int SB = 256;                            // tokens per inner block = threads
    __shared__ float q2[kMaxRep][kD];                  // q * sm_scale * log2(e)
    __shared__ float sc[kMaxRep][SB];                  // scores, then weights, of the inner block
    __shared__ float red[4][kMaxRep];                  // per-wave partial max / sum
    __shared__ float comb[kMaxRep][kD];

    const int u = blockIdx.y, ch = blockIdx.x, tid = threadIdx.x;
    const int b = u / a.Hkv, kvh = u % a.Hkv, rep = a.rep;
    const int bq0 = b * a.Hq + kvh * rep;
    const bool residual = (ch == a.nchunk);
    const int T = clampi(a.q_len[u], 0, a.Tcap);
    const int R = clampi(a.r_len[u], 0, a.Rcap);
    int t_begin, t_end;
    if (residual) { t_begin = 0; t_end = R; }
    else { t_begin = ch * a.chunk; t_end = min(T, t_begin + a.chunk); }
    if (t_begin >= t_end) return;                      // nothing here: the merge kernel skips this slot

    for (int i = tid; i < rep * kD; i += 256)
        q2[i / kD][i % kD] = hf(a.q[(size_t)(bq0 + i / kD) * kD + i % kD]) * a.c1;
    __syncthreads();

    const uint32_t *Kc = a.Kc + (size_t)u * kc_words(a.Tcap);
    const uint32_t *Vc = a.Vc + (size_t)u * vc_words(a.Tcap);
    const uint16_t *Ks = a.Ks + (size_t)u * (a.Tcap / G) * kD;
    const uint16_t *Kz = a.Kz + (size_t)u * (a.Tcap / G) * kD;
    const uint16_t *Vs = a.Vs + (size_t)u * a.Tcap * NCG;
    const uint16_t *Vz = a.Vz + (size_t)u * a.Tcap * NCG;
    const uint16_t *Rk = a.Rk + (size_t)u * a.Rcap * kD;
    const uint16_t *Rv = a.Rv + (size_t)u * a.Rcap * kD;

    float m[kMaxRep], l[kMaxRep], o[kMaxRep];
    for (int h = 0; h < kMaxRep; h++) { m[h] = -1e30f; l[h] = 0.f; o[h] = 0.f; }
    const int c = tid & (kD - 1), half = tid >> 7;

    for (int ts = t_begin; ts < t_end; ts += SB) {
        // ---- scores of token ts + tid for every query head of the group
        const int t = ts + tid;
        float acc[kMaxRep];
        for (int h = 0; h < kMaxRep; h++) acc[h] = 0.f;
        if (t < t_end) {
            if (!residual) {
                for (int w = 0; w < 8; w++) {
                    const uint32_t word = Kc[k_word_index(t, w)];
                    for (int k = 0; k < 16; k++) {
                        const int cc = 16 * w + k;
                        const float code = (float)((word >> k_bit(cc)) & 3u);
                        const size_t g = (size_t)(t / G) * kD + k_meta_pos(G, cc);
                        const float khat = code * hf(Ks[g]) + hf(Kz[g]);
                        for (int h = 0; h < rep; h++) acc[h] += q2[h][cc] * khat;
                    }
                }
            } else {
                for (int cc = 0; cc < kD; cc++) {
                    const float kv = hf(Rk[(size_t)t * kD + cc]);
                    for (int h = 0; h < rep; h++) acc[h] += q2[h][cc] * kv;
                }
            }
        }
        // ---- block max, weights, block sum
        for (int h = 0; h < rep; h++) {
            const float s = (t < t_end) ? acc[h] : -INFINITY;
            const float wm = wave_max(s);
            if ((tid & 63) == 0) red[tid >> 6][h] = wm;
            acc[h] = s;
        }
        __syncthreads();
        float scale[kMaxRep];
        for (int h = 0; h < rep; h++) {
            const float bm = fmaxf(fmaxf(red[0][h], red[1][h]), fmaxf(red[2][h], red[3][h]));
            const float mn = fmaxf(m[h], bm);
            scale[h] = exp2f(m[h] - mn);
            m[h] = mn;
            sc[h][tid] = exp2f(acc[h] - mn);           // exp2(-inf) = 0 for the masked tail
        }
        __syncthreads();
        for (int h = 0; h < rep; h++) {
            const float ws = wave_sum(sc[h][tid]);
            if ((tid & 63) == 0) red[tid >> 6][h] = ws;
        }
        __syncthreads();
        for (int h = 0; h < rep; h++) {
            l[h] = l[h] * scale[h] + (red[0][h] + red[1][h] + red[2][h] + red[3][h]);
            o[h] *= scale[h];
        }
        // ---- weighted values: thread (c, half) takes every other token of the block
        const int nb = min(SB, t_end - ts);
        for (int tt = half; tt < nb; tt += 2) {
            const int tv = ts + tt;
            float v;
            if (!residual) {
                const float code = (float)((Vc[v_word_index(tv >> 4, c)] >> v_bit(tv)) & 3u);
                const size_t g = (size_t)tv * NCG + c / G;
                v = code * hf(Vs[g]) + hf(Vz[g]);
            } else {
                v = hf(Rv[(size_t)tv * kD + c]);
            }
            for (int h = 0; h < rep; h++) o[h] += sc[h][tt] * v;
        }
        __syncthreads();
    }

    if (half == 1)
        for (int h = 0; h < rep; h++) comb[h][c] = o[h];
    __syncthreads();
    if (half == 0)
        for (int h = 0; h < rep; h++) {
            float *p = partial_ptr(a, bq0 + h, ch);
            p[4 + c] = o[h] + comb[h][c];
            if (c == 0) { p[0] = m[h]; p[1] = l[h]; }
        }
}

// One workgroup of 128 threads per query row: combine the valid partials and write fp16.
__global__ __launch_bounds__(128) void merge_kernel(DecArgs a)
{
    const int bq = blockIdx.x, c = threadIdx.x;
    const int b = bq / a.Hq, hq = bq % a.Hq;
    const int u = b * a.Hkv + hq / a.rep;
    const int T = clampi(a.q_len[u], 0, a.Tcap);
    const int R = clampi(a.r_len[u], 0, a.Rcap);
    const int nq = (T + a.chunk - 1) / a.chunk;

    float M = -1e30f;
    for (int ch = 0; ch < nq; ch++) M = fmaxf(M, partial_ptr(a, bq, ch)[0]);
    if (R > 0) M = fmaxf(M, partial_ptr(a, bq, a.nchunk)[0]);
    float L = 0.f, O = 0.f;
    for (int ch = 0; ch < nq; ch++) {
        const float *p = partial_ptr(a, bq, ch);
        const float w = exp2f(p[0] - M);
        L += p[1] * w;
        O += p[4 + c] * w;
    }
    if (R > 0) {
        const float *p = partial_ptr(a, bq, a.nchunk);
        const float w = exp2f(p[0] - M);
        L += p[1] * w;
        O += p[4 + c] * w;
    }
    const float r = (L > 0.f) ? O / L : 0.f;
    a.out[(size_t)bq * kD + c] = __half_as_ushort(__float2half_rn(r));
}

int launch_merge(const DecArgs &a, int nq, hipStream_t st)
{
    hipLaunchKernelGGL(merge_kernel, dim3(nq), dim3(128), 0, st, a);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

int launch_decode_scalar(const DecArgs &a, int G, int units, hipStream_t st)
{
    dim3 grid(a.nchunk + 1, units);
    switch (G) {
    case 16: hipLaunchKernelGGL(decode_scalar_kernel<16>, grid, dim3(256), 0, st, a); break;
    case 32: hipLaunchKernelGGL(decode_scalar_kernel<32>, grid, dim3(256), 0, st, a); break;
    case 64: hipLaunchKernelGGL(decode_scalar_kernel<64>, grid, dim3(256), 0, st, a); break;
    case 128: hipLaunchKernelGGL(decode_scalar_kernel<128>, grid, dim3(256), 0, st, a); break;
    default: return MINIKV_EUNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

int launch_decode(const minikv_shape &s, const minikv_f16 *q, const minikv_cache &c, float sm_scale,
                  minikv_f16 *out, void *workspace, int variant, hipStream_t st, const AppendArgs *ap)
{
    int *cnt = reinterpret_cast<int *>(workspace);
    return launch_decode_parts(s, q, c, sm_scale, out, cnt, cnt + ws_units(s), cnt + 3 * ws_units(s) + kMaxStreamWaves,
                               reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + ws_counter_bytes(s)),
                               variant, st, ap ? *ap : AppendArgs());
}

int launch_decode_parts(const minikv_shape &s, const minikv_f16 *q, const minikv_cache &c, float sm_scale,
                        minikv_f16 *out, int *cnt, int *cnt1, int *redo, float *partials, int variant, hipStream_t st,
                        const AppendArgs &ap)
{
    const DecodeGeom g = decode_geom(s);
    DecArgs a;
    a.q = q; a.Kc = c.Kc; a.Vc = c.Vc; a.Ks = c.Ks; a.Kz = c.Kz; a.Vs = c.Vs; a.Vz = c.Vz;
    a.Rk = c.Rk; a.Rv = c.Rv; a.q_len = c.q_len; a.r_len = c.r_len;
    a.out = out;
    a.append = ap.k_new != nullptr;
    a.k_new = ap.k_new; a.v_new = ap.v_new; a.r_len_out = ap.r_len_out;
    a.first_slot = 0;
    a.cnt = cnt;
    a.cnt1 = cnt1;
    a.redo = redo;
    a.ws = partials;
    a.c1 = sm_scale * 1.44269504088896340736f;
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.rep = g.rep; a.Tcap = s.Tcap; a.Rcap = s.Rcap;
    a.chunk = g.chunk; a.nchunk = g.nchunk;
    const int units = s.B * s.Hkv;
    a.units = units; a.hsets = (g.rep + 3) / 4;
    a.hs_shift = a.hsets > 1 ? 1 : 0;
    fast_div_setup((uint32_t)s.Hkv, a.hkv_magic, a.hkv_shift);
    int rc;
    if (variant == 0) variant = 3;                     // default variant
    if (a.append && variant != 3) return MINIKV_EUNSUPPORTED;   // the fused step exists in the default kernel only
    if (variant == 1) rc = launch_decode_scalar(a, s.G, units, st);
    else return launch_decode_tiled(a, s.G, units, variant, st);      // merges in the same launch
    if (rc) return rc;
    return launch_merge(a, s.B * s.Hq, st);
}

}  // namespace minikv
