// minikv_decode_attn_static: the decode attention call for callers that cannot allocate device memory
// (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  It runs the same kernel as
// minikv_decode_attn; the split-K workspace that call takes as an argument is here a file-scope device array.
#include "common.h"

#include <mutex>

namespace minikv {

// Largest number of (batch, KV head, set of four query heads) units the static workspace serves.
constexpr size_t kStaticUnits = 2048;
// Fixed layout, independent of the shape, so that calls with different shapes can follow each other: the
// ticket counters of the largest case first (they are zero between calls: the kernel returns every counter it
// used to zero), then the split-K partial slots (no initial state).
constexpr size_t kStaticCnt = kStaticUnits;                                   // per-unit counters
constexpr size_t kStaticCnt1 = 2 * kStaticUnits + kMaxStreamWaves;            // sub-group counters
constexpr size_t kStaticCounterBytes = ((kStaticCnt + kStaticCnt1 + 1) * sizeof(int) + 255) / 256 * 256;   // + the redo counter
constexpr size_t kStaticPartialBytes = ((size_t)kMaxStreamWaves + 2 * kStaticUnits) * 4 * kPartialStride * sizeof(float);
constexpr size_t kStaticBytes = kStaticCounterBytes + kStaticPartialBytes;    // about 17.3 MB per GPU

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// In host code `scratch` is only a handle for the runtime.  The address of each GPU's copy is looked up once,
// with that GPU current, and kept here.
constexpr int kMaxDevices = 64;
static std::mutex g_mutex;
static unsigned char *g_scratch_ptr[kMaxDevices];
static bool g_ready[kMaxDevices];

__global__ void fill_zero_kernel(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Device address of the current device's scratch array (null on failure).  On the first call for a device
// the counter part is also zero-filled on `st` (with a kernel, so that a capturing caller records no memset).
static unsigned char *scratch_of_current_device(hipStream_t st)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_ready[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(64), dim3(256), 0, st, reinterpret_cast<uint32_t *>(p),
                           kStaticCounterBytes / sizeof(uint32_t));
        if (hipGetLastError() != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = reinterpret_cast<unsigned char *>(p);
        g_ready[dev] = true;
    }
    return g_scratch_ptr[dev];
}

}  // namespace minikv

using namespace minikv;

extern "C" {

size_t minikv_static_workspace_units(void) { return kStaticUnits; }

int minikv_decode_attn_static(const minikv_shape *s, const minikv_f16 *q, const minikv_cache *c, float sm_scale,
                              minikv_f16 *out, void *stream)
{
    int rc = validate_shape(s);
    if (rc) return rc;
    if ((rc = validate_cache(*s, c))) return rc;
    if (!aligned16(q) || !aligned16(out)) return MINIKV_EINVAL;
    if (!(sm_scale == sm_scale) || sm_scale - sm_scale != 0.0f) return MINIKV_EINVAL;   // NaN / Inf
    if (ws_units(*s) > kStaticUnits) return MINIKV_EWORKSPACE;
    unsigned char *base = scratch_of_current_device((hipStream_t)stream);
    if (!base) return MINIKV_ELAUNCH;
    int *cnt = reinterpret_cast<int *>(base);
    return launch_decode_parts(*s, q, *c, sm_scale, out, cnt, cnt + kStaticCnt, cnt + kStaticCnt + kStaticCnt1,
                               reinterpret_cast<float *>(base + kStaticCounterBytes), 0, (hipStream_t)stream);
}

}  // extern "C"
