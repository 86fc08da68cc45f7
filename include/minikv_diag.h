/*
 * libminikv diagnostics -- entry points that serve measurements and cross-checks, not the decode path.
 * They are exported by the same shared library and follow the conventions of minikv.h (device pointers
 * owned by the caller, work enqueued on `stream`, negative minikv_status on a host-side check).
 */
#ifndef MINIKV_DIAG_H
#define MINIKV_DIAG_H

#include "minikv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* A plain streaming read (128-bit loads, 2048 workgroups) of `bytes` bytes (rounded down to 16) at src: the
 * reference point the bandwidth figures of the decode kernel are compared with.  sums: uint32 [2048] (device),
 * xor-updated with a checksum per workgroup. */
int minikv_stream_read_probe(const void *src, size_t bytes, uint32_t *sums, void *stream);

/* How many (wave, unit) pairs minikv_decode_attn has redone with range-normalised operands since `workspace` was
 * zero-filled (the second attempt taken when an fp16 matrix operand overflowed, see minikv.h): 0 for data inside
 * the fast range.  Synchronous (a blocking 4-byte copy to the host); count is a HOST pointer. */
int minikv_diag_redo_count(const minikv_shape *shape, const void *workspace, int32_t *count);

/* How minikv_decode_attn / minikv_decode_step cut the work into waves (process-wide): 0 = chosen by shape
 * (default), 1 = a residual item of 64 tokens weighs 3.5 quantized passes of 128, as measured (what large launches
 * use), 2 = every item weighs the same (what launches of few items use, so that every item gets a wave).  Both
 * give the same result up to the order of the merge; the parity tests run each.  MINIKV_EINVAL otherwise. */
int         minikv_diag_decode_weights(int mode);

/* Which kernels kv_select_hh_rw launches (process-wide): 0 = chosen by shape (default), 1 = always one workgroup
 * per unit, 2 = several workgroups per unit whenever the prompt has at most 1024 chunks of 4096 tokens.  Both
 * give the same positions; the parity tests run each.  MINIKV_EINVAL for any other value. */
int         minikv_diag_select_path(int path);

/* Selects the kernel minikv_decode_attn launches (process-wide):
 *   0 = default, 1 = a plain scalar-loop fp32 kernel (two launches) kept as a second GPU implementation of
 *   Algorithm 1 lines 17-19 for cross-checks, 3 = the default kernel by its own number.
 * Returns MINIKV_EINVAL for any other id.  minikv_strvariant names an id. */
int         minikv_set_variant(int variant);
const char *minikv_strvariant(int variant);

#ifdef __cplusplus
}
#endif
#endif
