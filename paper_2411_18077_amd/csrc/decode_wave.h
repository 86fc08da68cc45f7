// Wave-level building blocks shared by the decode-attention kernels (gfx950, wave64): code-field
// extraction as fp16 subnormals, DPP reductions, the 4x4x4 matrix instruction with operand broadcast,
// the per-pass register tiles, device-scope loads and stores for the split-K partials.
#pragma once

#include "decode_common.h"

#include <hip/hip_fp16.h>

namespace minikv {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

constexpr int kNH = 4;                 // query-head slots per workgroup (rows of the 4x4x4 blocks)
constexpr int kPass = 128;             // tokens per wave pass
constexpr int kPsH = kPass + 4;        // halfs per (channel group, head) row of ps, padded
constexpr int kPsG = kNH * kPsH;       // halfs per channel group of ps (528: shifts 8 banks)
constexpr int kKRowH = kD + 8;         // halfs per staged residual key row (272 B: rows start 4 banks apart)

__device__ inline h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ inline uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// field j (0..7) of a half-word pair -> (shift inside the mantissa, use the >>6 copy?)
__host__ __device__ constexpr int fld_shift(int j) { return j <= 4 ? 2 * j : 2 * (j - 3); }
__host__ __device__ constexpr bool fld_shifted(int j) { return j > 4; }
// 4^-(shift/2): what the small operand is pre-multiplied by so that the masked subnormal needs no shift
__device__ inline float fld_scale(int j) { return 1.0f / (float)(1 << fld_shift(j)); }

__device__ inline h2 field(uint32_t w, uint32_t w6, int j)
{
    return as_h2((fld_shifted(j) ? w6 : w) & (0x00030003u << fld_shift(j)));
}

// ---- cross-lane reductions on the DPP data path (no LDS traffic)
template <int CTRL, int ROW_MASK = 0xF>
__device__ inline float dpp_mov(float old, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v),
                                                                  CTRL, ROW_MASK, 0xF, false));
}

// Four independent reductions at once, hand-scheduled: step k of all four values is issued back to back,
// so the two wait states a DPP read needs after a VALU write are always covered by the other three.
#define MINIKV_DPP4(op, ctrl)                                                     \
    "v_" op "_f32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %2, %2, %2 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %3, %3, %3 " ctrl " bank_mask:0xf\n"
#define MINIKV_ROW16(op)                                                          \
    MINIKV_DPP4(op, "quad_perm:[1,0,3,2] row_mask:0xf")                           \
    MINIKV_DPP4(op, "quad_perm:[2,3,0,1] row_mask:0xf")                           \
    MINIKV_DPP4(op, "row_half_mirror row_mask:0xf")                               \
    MINIKV_DPP4(op, "row_mirror row_mask:0xf")
#define MINIKV_WAVE64(op)                                                         \
    MINIKV_ROW16(op)                                                              \
    MINIKV_DPP4(op, "row_bcast:15 row_mask:0xa")                                  \
    MINIKV_DPP4(op, "row_bcast:31 row_mask:0xc")

__device__ inline float lane63(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// v[i] <- maximum of v[i] over the wave (wave-uniform)
__device__ inline void wave_max64x4(float v[4])
{
    asm volatile("s_nop 1\n" MINIKV_WAVE64("max") : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
    for (int i = 0; i < 4; i++) v[i] = lane63(v[i]);
}
// the same for two values (the wait states between dependent DPP steps are filled with s_nop)
#define MINIKV_DPP2(op, ctrl)                                                     \
    "v_" op "_f32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n"                        \
    "v_" op "_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n"                        \
    "s_nop 0\n"
#define MINIKV_WAVE64X2(op)                                                       \
    MINIKV_DPP2(op, "quad_perm:[1,0,3,2] row_mask:0xf")                           \
    MINIKV_DPP2(op, "quad_perm:[2,3,0,1] row_mask:0xf")                           \
    MINIKV_DPP2(op, "row_half_mirror row_mask:0xf")                               \
    MINIKV_DPP2(op, "row_mirror row_mask:0xf")                                    \
    MINIKV_DPP2(op, "row_bcast:15 row_mask:0xa")                                  \
    MINIKV_DPP2(op, "row_bcast:31 row_mask:0xc")
__device__ inline void wave_max64x2(float v[2])
{
    asm volatile("s_nop 1\n" MINIKV_WAVE64X2("max") : "+v"(v[0]), "+v"(v[1]));
    for (int i = 0; i < 2; i++) v[i] = lane63(v[i]);
}
// v[i] <- sum of v[i] over the wave (wave-uniform)
__device__ inline void wave_sum64x4(float v[4])
{
    asm volatile("s_nop 1\n" MINIKV_WAVE64("add") : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
    for (int i = 0; i < 4; i++) v[i] = lane63(v[i]);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; exp2(-inf) = 0

template <int N> struct Words { uint32_t v[N]; };
template <int N> __device__ inline Words<N> load_words(const void *p)
{
    Words<N> r;
    if constexpr (N == 1) { r.v[0] = *reinterpret_cast<const uint32_t *>(p); }
    else if constexpr (N == 2) { uint2 t = *reinterpret_cast<const uint2 *>(p); r.v[0] = t.x; r.v[1] = t.y; }
    else {
        for (int i = 0; i < N / 4; i++) {
            uint4 t = reinterpret_cast<const uint4 *>(p)[i];
            r.v[4 * i] = t.x; r.v[4 * i + 1] = t.y; r.v[4 * i + 2] = t.z; r.v[4 * i + 3] = t.w;
        }
    }
    return r;
}

// The broadcast controls of the matrix instruction are immediates; these helpers turn the (unrolled,
// hence constant) block index into one.
#define MINIKV_MFMA_CASE(n) case n: acc = __builtin_amdgcn_mfma_f32_4x4x4f16(av, bv, acc, CB, n, 0); break;
template <int CB>
__device__ inline void mfma_bc(f4 &acc, h4 av, h4 bv, int abid)
{
    switch (abid) {
        MINIKV_MFMA_CASE(0) MINIKV_MFMA_CASE(1) MINIKV_MFMA_CASE(2) MINIKV_MFMA_CASE(3)
        MINIKV_MFMA_CASE(4) MINIKV_MFMA_CASE(5) MINIKV_MFMA_CASE(6) MINIKV_MFMA_CASE(7)
        MINIKV_MFMA_CASE(8) MINIKV_MFMA_CASE(9) MINIKV_MFMA_CASE(10) MINIKV_MFMA_CASE(11)
        MINIKV_MFMA_CASE(12) MINIKV_MFMA_CASE(13) MINIKV_MFMA_CASE(14) MINIKV_MFMA_CASE(15)
    }
}
template <int CB>
__device__ inline void mfma_k(f4 &acc0, f4 &acc1, h4 av, h4 b0, h4 b1, int abid)
{
    mfma_bc<CB>(acc0, av, b0, abid);
    mfma_bc<CB>(acc1, av, b1, abid);
}
template <int CB>
__device__ inline void mfma_v(f4 &o0, f4 &o1, h4 a0, h4 a1, h4 b0, h4 b1, int abid)
{
    mfma_bc<CB>(o0, a0, b0, abid);
    mfma_bc<CB>(o1, a1, b1, abid);
}

// ------------------------------------------------------------------------------------------------
constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }

template <int N>
__device__ inline float dpp_ror_add(float v)              // v + (v rotated right by N lanes inside its row of 16)
{
    return v + dpp_mov<0x120 + N>(0.f, v);
}
template <int H>
__device__ inline float quad_bcast(float v)               // value of lane (4*(lane/4) + H)
{
    return dpp_mov<H * 0x55>(0.f, v);
}

// What one wave needs from global memory for the K half and the V half of one pass of 128 tokens.
template <int NKW>
struct KData {
    u4 kw[4];               // K code words of tokens 2*lane (kw[0..1]) and 2*lane+1 (kw[2..3])
    Words<NKW> ks, kz;      // this lane's bin of the K scale / zero row of its group
};
template <int NCG>
struct VData {
    u4 vw[2][2];            // V code words [channel lane / lane+64][64-token tile]: 4 blocks of 16 tokens each
    Words<NCG> vs, vz;      // V scale / zero of tokens 2*lane and 2*lane+1 (zero when past the end)
};

// Split-K partials travel between workgroups (possibly on different XCDs, each with its own L2) inside
// one launch.  They are written and read with device-scope relaxed atomics, which the hardware performs
// at the device-coherent level instead of in the XCD-local L2, so no L2 write-back or invalidate is needed;
// the writer only has to wait for its stores to be acknowledged before it takes the ticket.
__device__ inline float ld_agent(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float2 ld_agent2(const float *p)      // two consecutive floats, p 8-byte aligned
{
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return float2{__builtin_bit_cast(float, (uint32_t)v), __builtin_bit_cast(float, (uint32_t)(v >> 32))};
}
__device__ inline void st_agent(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent_i32(int *p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace minikv
