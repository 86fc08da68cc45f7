// Host side of libminikv: argument checks, buffer sizes, launch geometry, C entry points.
#include "common.h"
#include "minikv_diag.h"

#include <atomic>

namespace minikv {

static std::atomic<int> g_variant{0};

int validate_shape(const minikv_shape *s)
{
    if (!s) return MINIKV_EINVAL;
    if (s->D != kD) return MINIKV_EUNSUPPORTED;
    if (!(s->G == 16 || s->G == 32 || s->G == 64 || s->G == 128)) return MINIKV_EUNSUPPORTED;
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv) return MINIKV_EINVAL;
    if (s->Hq / s->Hkv > kMaxRep) return MINIKV_EUNSUPPORTED;
    if (s->Tcap <= 0 || s->Tcap % kKTile) return MINIKV_EINVAL;
    if (s->Rcap < 0 || s->Rcap % s->G) return MINIKV_EINVAL;
    if ((int64_t)s->B * s->Hkv > 65535) return MINIKV_EINVAL;      // units index a grid dimension
    return MINIKV_OK;
}

DecodeGeom decode_geom(const minikv_shape &s)
{
    // Token chunks of the cross-check kernel (the single-launch kernel balances by itself): enough
    // workgroups to cover the chip several times over, but no smaller than kMinChunk.
    const long units = (long)s.B * s.Hkv;
    int chunk = kMinChunk;
    while (chunk < 4096 && units * ((s.Tcap + 2 * chunk - 1) / (2 * chunk)) >= 2048) chunk *= 2;
    DecodeGeom g;
    g.chunk = chunk;
    g.nchunk = (s.Tcap + chunk - 1) / chunk;
    g.rep = s.Hq / s.Hkv;
    return g;
}

bool aligned16(const void *p) { return p && ((uintptr_t)p & 15u) == 0; }

int validate_cache(const minikv_shape &s, const minikv_cache *c)
{
    if (!c) return MINIKV_EINVAL;
    if (!aligned16(c->Kc) || !aligned16(c->Ks) || !aligned16(c->Kz) || !aligned16(c->Vc) ||
        !aligned16(c->Vs) || !aligned16(c->Vz) || !c->q_len || !c->r_len)
        return MINIKV_EINVAL;
    if (s.Rcap > 0 && (!aligned16(c->Rk) || !aligned16(c->Rv))) return MINIKV_EINVAL;
    return MINIKV_OK;
}

// Reference point for the bandwidth figures: reads a buffer once with 128-bit loads, 2048 workgroups striding
// through it, and folds it into one word per workgroup (so that the loads cannot be dropped).
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ src, size_t n16,
                                                         uint32_t *__restrict__ sums)
{
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256 * 8;
    for (size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x; i < n16; i += stride) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const size_t k = i + (size_t)j * 256;
            v[j] = src[k < n16 ? k : n16 - 1];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    for (int d = 32; d >= 1; d >>= 1) acc ^= __shfl_xor(acc, d, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(&sums[blockIdx.x], acc);
}

}  // namespace minikv

using namespace minikv;

extern "C" {

int minikv_abi_version(void) { return MINIKV_ABI_VERSION; }

const char *minikv_strerror(int status)
{
    switch (status) {
    case MINIKV_OK: return "ok";
    case MINIKV_EINVAL: return "invalid argument (null or misaligned pointer, or a shape rule violated)";
    case MINIKV_EUNSUPPORTED: return "unsupported shape (D must be 128, G in {16,32,64,128}, Hq/Hkv <= 8)";
    case MINIKV_EWORKSPACE: return "workspace too small (see minikv_workspace_bytes)";
    case MINIKV_ELAUNCH: return "HIP launch failed";
    default: return "unknown status";
    }
}

size_t minikv_cache_bytes(const minikv_shape *s, int which) { return minikv_buffer_bytes(s, which); }

size_t minikv_buffer_bytes(const minikv_shape *s, int which)
{
    if (validate_shape(s) != MINIKV_OK) return 0;
    const size_t U = (size_t)s->B * s->Hkv;
    switch (which) {
    case MINIKV_BUF_KC: return U * kc_words(s->Tcap) * 4;
    case MINIKV_BUF_KS:
    case MINIKV_BUF_KZ: return U * (size_t)(s->Tcap / s->G) * kD * 2;
    case MINIKV_BUF_VC: return U * vc_words(s->Tcap) * 4;
    case MINIKV_BUF_VS:
    case MINIKV_BUF_VZ: return U * (size_t)s->Tcap * (kD / s->G) * 2;
    case MINIKV_BUF_QLEN:
    case MINIKV_BUF_RLEN: return U * 4;
    case MINIKV_BUF_RK:
    case MINIKV_BUF_RV: return U * (size_t)s->Rcap * kD * 2;
    default: return 0;
    }
}

size_t minikv_workspace_bytes(const minikv_shape *s)
{
    if (validate_shape(s) != MINIKV_OK) return 0;
    // cross-check kernel: one partial per (query row, chunk) for the smallest chunk, plus the residual chunk
    const size_t nch = (size_t)(s->Tcap + kMinChunk - 1) / kMinChunk + 1;
    const size_t scalar = (size_t)s->B * s->Hq * nch * kPartialStride * sizeof(float);
    // single-launch kernel: one slot of 4 heads per (wave, unit it serves): slot = wave + 2 * unit
    const size_t nu = ws_units(*s);
    const size_t stream = ((size_t)kMaxStreamWaves + 2 * nu) * 4 * kPartialStride * sizeof(float);
    return ws_counter_bytes(*s) + (scalar > stream ? scalar : stream);
}

int kv_quantize_pack(const minikv_shape *s, const minikv_f16 *K, const minikv_f16 *V, int64_t L,
                     const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, int32_t max_tok,
                     minikv_cache *c, void *stream)
{
    int rc = validate_shape(s);
    if (rc) return rc;
    if ((rc = validate_cache(*s, c))) return rc;
    if (!aligned16(K) || !aligned16(V) || !n_tok || L <= 0) return MINIKV_EINVAL;
    if (max_tok < 0 || max_tok % s->G || max_tok > s->Tcap || max_tok > L) return MINIKV_EINVAL;
    if (idx && idx_stride < max_tok) return MINIKV_EINVAL;
    if (max_tok == 0) return MINIKV_OK;
    return launch_quantize(*s, K, V, L, idx, idx_stride, n_tok, max_tok, *c, false, (hipStream_t)stream);
}

int kv_flush_residual(const minikv_shape *s, minikv_cache *c, void *stream)
{
    int rc = validate_shape(s);
    if (rc) return rc;
    if ((rc = validate_cache(*s, c))) return rc;
    if (s->Rcap == 0) return MINIKV_OK;
    if (s->Rcap > s->Tcap) return MINIKV_EINVAL;
    return launch_quantize(*s, c->Rk, c->Rv, s->Rcap, nullptr, 0, c->r_len, s->Rcap, *c, true,
                           (hipStream_t)stream);
}

int kv_append_residual(const minikv_shape *s, const minikv_f16 *k_new, const minikv_f16 *v_new,
                       minikv_cache *c, void *stream)
{
    int rc = validate_shape(s);
    if (rc) return rc;
    if ((rc = validate_cache(*s, c))) return rc;
    if (!aligned16(k_new) || !aligned16(v_new)) return MINIKV_EINVAL;
    if (s->Rcap == 0) return MINIKV_EINVAL;
    return launch_append(*s, k_new, v_new, *c, (hipStream_t)stream);
}

int minikv_decode_attn(const minikv_shape *s, const minikv_f16 *q, const minikv_cache *c, float sm_scale,
                       minikv_f16 *out, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = validate_shape(s);
    if (rc) return rc;
    if ((rc = validate_cache(*s, c))) return rc;
    if (!aligned16(q) || !aligned16(out) || !aligned16(workspace)) return MINIKV_EINVAL;
    if (!(sm_scale == sm_scale) || sm_scale - sm_scale != 0.0f) return MINIKV_EINVAL;   // NaN / Inf
    if (workspace_bytes < minikv_workspace_bytes(s)) return MINIKV_EWORKSPACE;
    return launch_decode(*s, q, *c, sm_scale, out, workspace, g_variant.load(), (hipStream_t)stream);
}

int minikv_decode_step(const minikv_shape *s, const minikv_f16 *q, const minikv_f16 *k_new, const minikv_f16 *v_new,
                       const minikv_cache *c, int32_t *r_len_next, float sm_scale, minikv_f16 *out, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    int rc = validate_shape(s);
    if (rc) return rc;
    if ((rc = validate_cache(*s, c))) return rc;
    if (!aligned16(q) || !aligned16(out) || !aligned16(workspace) || !aligned16(k_new) || !aligned16(v_new))
        return MINIKV_EINVAL;
    if (!k_new || !v_new || !r_len_next || ((uintptr_t)r_len_next & 3u) || r_len_next == c->r_len) return MINIKV_EINVAL;
    if (!(sm_scale == sm_scale) || sm_scale - sm_scale != 0.0f) return MINIKV_EINVAL;   // NaN / Inf
    if (workspace_bytes < minikv_workspace_bytes(s)) return MINIKV_EWORKSPACE;
    AppendArgs ap;
    ap.k_new = k_new, ap.v_new = v_new, ap.r_len_out = r_len_next;
    return launch_decode(*s, q, *c, sm_scale, out, workspace, 0, (hipStream_t)stream, &ap);
}

size_t selective_flash_attn_workspace_bytes(int32_t B, int32_t Hkv, int64_t L)
{
    if (B <= 0 || Hkv <= 0 || L < 1) return 0;
    return (size_t)B * Hkv * kD * (size_t)((L + 63) / 64 * 64) * sizeof(minikv_f16);     // V transposed, keys padded to 64
}

int selective_flash_attn(int32_t B, int32_t Hq, int32_t Hkv, int64_t L, const minikv_f16 *Q, const minikv_f16 *K,
                         const minikv_f16 *V, float sm_scale, minikv_f16 *X_O, float *lse, float *A_cumul,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || L < 1 || L > ((int64_t)1 << 23)) return MINIKV_EINVAL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(X_O) || !aligned16(lse)) return MINIKV_EINVAL;
    if (A_cumul && ((uintptr_t)A_cumul & 15u)) return MINIKV_EINVAL;
    if (!aligned16(workspace)) return MINIKV_EINVAL;
    if (!(sm_scale > 0.0f) || sm_scale - sm_scale != 0.0f) return MINIKV_EINVAL;       // positive and finite
    if ((int64_t)B * Hq * ((L + 127) / 128) > 0x7fffffff || (int64_t)B * Hkv > 65535) return MINIKV_EINVAL;
    if (workspace_bytes < selective_flash_attn_workspace_bytes(B, Hkv, L)) return MINIKV_EWORKSPACE;
    return launch_prefill(B, Hq, Hkv, L, Q, K, V, sm_scale, X_O, lse, A_cumul, workspace, (hipStream_t)stream);
}

size_t kv_select_workspace_bytes(int32_t units, int32_t rep, int64_t L)
{
    return select_workspace_bytes(units, rep, L);
}

int kv_select_hh_rw(int32_t units, int32_t rep, int64_t L, const float *A_cumul, const int32_t *n_hh,
                    const int32_t *n_rw, int32_t *idx, int64_t idx_stride, int32_t *n_tok, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    if (units < 0 || rep < 1 || L < 0 || L > ((int64_t)1 << 30) || idx_stride < 0) return MINIKV_EINVAL;
    if (units == 0) return MINIKV_OK;
    if (!n_hh || !n_rw || !idx || !n_tok || ((uintptr_t)idx & 3u) || ((uintptr_t)n_tok & 3u)) return MINIKV_EINVAL;
    if (L > 0 && (!A_cumul || ((uintptr_t)A_cumul & 3u))) return MINIKV_EINVAL;
    const size_t need = kv_select_workspace_bytes(units, rep, L);
    if (need && (!workspace || ((uintptr_t)workspace & 15u))) return MINIKV_EINVAL;
    if (workspace_bytes < need) return MINIKV_EWORKSPACE;
    return launch_select(units, rep, L, A_cumul, n_hh, n_rw, idx, idx_stride, n_tok, workspace,
                         (hipStream_t)stream);
}

int kv_pyramid_budget(int32_t n_layers, double x, int32_t d, int32_t bottom_heavy, double *budget)
{
    if (n_layers < 1 || d < 1 || !(x >= 0.0) || !budget) return MINIKV_EINVAL;
    // The budgets are symmetric about x: layer l holds x + t * (x - x/d) with t running from -1 at one end
    // layer to +1 at the other, so the ends are x/d and 2x - x/d and the mean is x.
    const double half_range = x - x / (double)d;
    for (int32_t l = 0; l < n_layers; ++l) {
        const double t = n_layers == 1 ? 0.0 : (2.0 * l - (n_layers - 1)) / (double)(n_layers - 1);
        budget[l] = x + (bottom_heavy ? -t : t) * half_range;
    }
    return MINIKV_OK;
}

int minikv_stream_read_probe(const void *src, size_t bytes, uint32_t *sums, void *stream)
{
    if (!aligned16(src) || !sums || ((uintptr_t)sums & 3u) || bytes < 16) return MINIKV_EINVAL;
    hipLaunchKernelGGL(stream_read_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src,
                       bytes / 16, sums);
    return hipGetLastError() == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

int minikv_diag_redo_count(const minikv_shape *s, const void *workspace, int32_t *count)
{
    if (validate_shape(s) != MINIKV_OK || !workspace || !count) return MINIKV_EINVAL;
    const int *p = reinterpret_cast<const int *>(workspace) + 3 * ws_units(*s) + kMaxStreamWaves;
    return hipMemcpy(count, p, sizeof(int32_t), hipMemcpyDeviceToHost) == hipSuccess ? MINIKV_OK : MINIKV_ELAUNCH;
}

int minikv_diag_decode_weights(int mode)
{
    return set_decode_weights(mode) ? MINIKV_OK : MINIKV_EINVAL;
}

int minikv_diag_select_path(int path)
{
    return set_select_path(path) ? MINIKV_OK : MINIKV_EINVAL;
}

int minikv_set_variant(int variant)
{
    if (!(variant == 0 || variant == 1 || variant == 3)) return MINIKV_EINVAL;
    g_variant.store(variant);
    return MINIKV_OK;
}

const char *minikv_strvariant(int variant)
{
    switch (variant) {
    case 0: return "default";
    case 1: return "scalar: plain per-token loops, fp32 FMA (cross-check kernel)";
    case 3: return "wave-tiled, 4x4x4 fp16 matrix-core blocks for the head x channel products";
    default: return "unknown";
    }
}

}  // extern "C"
