// Internal declarations shared by the translation units of libminikv (GPU library only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "minikv.h"

namespace minikv {

constexpr int kD = 128;            // head dimension (the only one supported)
constexpr int kKTile = 128;        // tokens per K code tile (1024 words)
constexpr int kVTile = 64;         // tokens per V code tile (4*D words)
constexpr int kPartialStride = 132;  // floats per split-K partial: m, l, 2 pad, o[128]
constexpr int kMinChunk = 512;     // smallest token chunk one workgroup of the decode kernel takes
constexpr int kMaxRep = 8;         // most query heads per KV head
constexpr int kMaxStreamWaves = 4096;  // most single-wave workgroups the decode kernel is launched with

// Workspace layout of the single-launch decode kernel: ticket counters (zero between calls) -- one per
// (unit, set of 4 query heads) and one per partial slot for the sub-groups of 16 waves -- then the split-K
// partials (slot = wave + 2 * unit, fewer than kMaxStreamWaves + 2 * units of them).  One more word behind the
// ticket counters counts the units that had to be redone with range-normalised operands (never reset by the
// kernels; read by minikv_diag_redo_count).
__host__ __device__ inline size_t ws_units(const minikv_shape &s)
{
    return (size_t)s.B * s.Hkv * ((s.Hq / s.Hkv + 3) / 4);
}
__host__ __device__ inline size_t ws_counter_bytes(const minikv_shape &s)
{
    return ((3 * ws_units(s) + kMaxStreamWaves + 1) * sizeof(int) + 255) / 256 * 256;
}

// per-unit element counts
__host__ __device__ inline size_t kc_words(int Tcap) { return (size_t)Tcap / kKTile * 1024; }
__host__ __device__ inline size_t vc_words(int Tcap) { return (size_t)Tcap / kVTile * 4 * kD; }

// Word index (inside one unit's Kc) of word w (0..7) of token t.
__host__ __device__ inline uint32_t k_word_index(int t, int w)
{
    int tile = t >> 7, tau = t & 127;
    return (uint32_t)tile * 1024u + (uint32_t)(((2 * (tau & 1) + (w >> 2)) * 64 + (tau >> 1)) * 4 + (w & 3));
}
// Bit position of channel c inside its K word.
__host__ __device__ inline int k_bit(int c) { return 16 * (c & 1) + 2 * ((c & 15) >> 1); }

// Position of channel c inside a K scale / zero row: the 32 channel quads are dealt round-robin into
// NB = G/8 bins so that every lane of the decode kernel finds its quads contiguous.
__host__ __device__ inline int k_meta_pos(int G, int c)
{
    const int nb = G >> 3, q = c >> 2;
    return ((q % nb) * (32 / nb) + q / nb) * 4 + (c & 3);
}

// Word index (inside one unit's Vc) of the 16-token block tb = t/16 of channel c.
__host__ __device__ inline uint32_t v_word_index(int tb, int c)
{
    return (uint32_t)(tb >> 2) * (4u * kD) + (uint32_t)c * 4u + (uint32_t)(tb & 3);
}
// Bit position of token t inside its V word.
__host__ __device__ inline int v_bit(int t) { return 16 * (t & 1) + 2 * ((t & 15) >> 1); }

// Decode launch geometry, derived from the shape alone so that the main kernel, the merge kernel and
// minikv_workspace_bytes() agree.
struct DecodeGeom {
    int chunk;      // quantized tokens per workgroup
    int nchunk;     // quantized-token chunks per unit (Tcap / chunk, rounded up)
    int rep;        // query heads per KV head
};
DecodeGeom decode_geom(const minikv_shape &s);

int validate_shape(const minikv_shape *s);

// launchers (one per translation unit)
int launch_quantize(const minikv_shape &s, const minikv_f16 *K, const minikv_f16 *V, int64_t L,
                    const int32_t *idx, int64_t idx_stride, const int32_t *n_tok, int32_t max_tok,
                    const minikv_cache &c, bool flush, hipStream_t st);
int launch_append(const minikv_shape &s, const minikv_f16 *k_new, const minikv_f16 *v_new,
                  const minikv_cache &c, hipStream_t st);
// the new token's rows and where the lengths after the append go: all null for plain attention
struct AppendArgs {
    const minikv_f16 *k_new = nullptr, *v_new = nullptr;
    int32_t *r_len_out = nullptr;
};
int launch_decode(const minikv_shape &s, const minikv_f16 *q, const minikv_cache &c, float sm_scale,
                  minikv_f16 *out, void *workspace, int variant, hipStream_t st, const AppendArgs *ap = nullptr);

// the same with the three parts of the workspace given one by one: per-unit ticket counters (ws_units ints),
// sub-group ticket counters (2 * ws_units + kMaxStreamWaves ints), the redo counter (one int), split-K partials
int launch_decode_parts(const minikv_shape &s, const minikv_f16 *q, const minikv_cache &c, float sm_scale,
                        minikv_f16 *out, int *cnt, int *cnt1, int *redo, float *partials, int variant, hipStream_t st,
                        const AppendArgs &ap = AppendArgs());
int validate_cache(const minikv_shape &s, const minikv_cache *c);
bool aligned16(const void *p);

int launch_prefill(int32_t B, int32_t Hq, int32_t Hkv, int64_t L, const minikv_f16 *Q, const minikv_f16 *K,
                   const minikv_f16 *V, float sm_scale, minikv_f16 *XO, float *lse, float *A_cumul,
                   void *workspace, hipStream_t st);
size_t select_workspace_bytes(int32_t units, int32_t rep, int64_t L);
bool set_decode_weights(int mode); // 0 = by shape, 1 = measured item weights, 2 = unit weights
bool set_select_path(int path);   // 0 = by shape, 1 = one workgroup per unit, 2 = several (when the prompt allows)
int launch_select(int32_t units, int32_t rep, int64_t L, const float *A, const int32_t *n_hh,
                  const int32_t *n_rw, int32_t *idx, int64_t idx_stride, int32_t *n_tok, void *workspace,
                  hipStream_t st);

}  // namespace minikv
