// Measurement aids (not steps of the method): a register-resident bf16 MFMA loop that shows what the
// matrix pipe sustains on this chip, and a plain copy kernel of known size used to calibrate the
// memory-traffic counters of the profiler.
#include "common.h"

namespace astraea {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// 4 independent accumulator chains of v_mfma_f32_32x32x16_bf16 per wave, operands held in registers.
// With random operands the chip runs into its power limit and lowers the clock; with constant
// operands it does not, so both are reported.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float *sink, int iters, int randomize)
{
    bf16x8 a[4], b[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t h = mix(threadIdx.x * 131u + blockIdx.x * 7919u + k * 17u + j);
            a[k][j] = (__bf16)(randomize ? ((h & 0xffff) / 32768.0f - 1.0f) : 1.0f);
            b[k][j] = (__bf16)(randomize ? (((h >> 16) & 0xffff) / 32768.0f - 1.0f) : 1.0f);
        }
    floatx16 c0, c1, c2, c3;
#pragma unroll
    for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// One 16-byte vector per thread, streaming load and store: the fastest plain copy found on this chip
// (6.2 - 6.6 TB/s read + write for 1 GiB; a grid-stride loop over 4096 workgroups reaches 4.6, eight vectors per
// thread 5.4, the runtime's device-to-device copy 4.9).
__global__ __launch_bounds__(256) void copy_kernel(const uint4v *__restrict__ src, uint4v *__restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace
}  // namespace astraea

using namespace astraea;

extern "C" {

int astraea_probe_mfma_bf16(int32_t workgroups, int32_t iters, int32_t randomize, float *sink, int64_t sink_elems,
                            double *flops_out, void *stream)
{
    if (workgroups <= 0 || iters <= 0 || !sink || sink_elems < (int64_t)workgroups * 256)
        return fail(ASTRAEA_ERR_INVALID, "astraea_probe_mfma_bf16: sink must hold workgroups*256 floats");
    hipLaunchKernelGGL(mfma_loop_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream, sink, iters,
                       randomize);
    // 4 waves per workgroup, 4 MFMAs per iteration, 2*32*32*16 flops each
    if (flops_out) *flops_out = (double)workgroups * 4.0 * (double)iters * 4.0 * 32768.0;
    return check_launch("astraea_probe_mfma_bf16");
}

int astraea_probe_copy(const void *src, void *dst, int64_t bytes, void *stream)
{
    if (bytes < 0 || bytes % 16 != 0 || ((uintptr_t)src | (uintptr_t)dst) % 16 != 0)
        return fail(ASTRAEA_ERR_INVALID, "astraea_probe_copy: pointers and size must be multiples of 16 bytes");
    if (bytes == 0) return ASTRAEA_OK;
    if (!src || !dst) return fail(ASTRAEA_ERR_INVALID, "astraea_probe_copy: NULL pointer");
    const size_t n = (size_t)(bytes / 16);
    if ((n + 255) / 256 > 2147483647ull) return fail(ASTRAEA_ERR_INVALID, "astraea_probe_copy: more than 8 TiB");
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (const uint4v *)src,
                       (uint4v *)dst, n);
    return check_launch("astraea_probe_copy");
}

}  // extern "C"

// ---- kernel timer: events around the attention's main kernel, kept per thread ----
namespace astraea {
namespace {
constexpr int kTimerSlots = 64;
struct KernelTimer {
    bool enabled = false;
    bool open = false;       // a begin without its end yet
    int count = 0;           // completed pairs
    bool created = false;
    hipEvent_t ev[kTimerSlots][2];
};
thread_local KernelTimer g_timer;
}  // namespace

void kernel_timer_begin(hipStream_t stream)
{
    KernelTimer &t = g_timer;
    if (!t.enabled || t.count >= kTimerSlots) return;
    // under stream capture an event record would become a graph node with no time of its own: skip the launch
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return;
    if (hipEventRecord(t.ev[t.count][0], stream) == hipSuccess) t.open = true;
}
void kernel_timer_end(hipStream_t stream)
{
    KernelTimer &t = g_timer;
    if (!t.open) return;
    t.open = false;
    if (hipEventRecord(t.ev[t.count][1], stream) == hipSuccess) ++t.count;
}
}  // namespace astraea

extern "C" int astraea_probe_kernel_timer(int enable)
{
    using namespace astraea;
    KernelTimer &t = g_timer;
    if (enable && !t.created) {
        for (int i = 0; i < kTimerSlots; ++i)
            for (int j = 0; j < 2; ++j)
                if (hipEventCreate(&t.ev[i][j]) != hipSuccess)
                    return fail(ASTRAEA_ERR_HIP, "astraea_probe_kernel_timer: hipEventCreate failed");
        t.created = true;
    }
    t.enabled = enable != 0;
    t.open = false;
    t.count = 0;
    return ASTRAEA_OK;
}

extern "C" int astraea_probe_kernel_ms(int32_t index, double *ms_out)
{
    using namespace astraea;
    KernelTimer &t = g_timer;
    if (!ms_out) return fail(ASTRAEA_ERR_INVALID, "astraea_probe_kernel_ms: NULL output");
    if (index < 0 || index >= t.count)
        return fail(ASTRAEA_ERR_INVALID, "astraea_probe_kernel_ms: %d launches were timed, index %d asked", t.count,
                    (int)index);
    if (hipEventSynchronize(t.ev[index][1]) != hipSuccess)
        return fail(ASTRAEA_ERR_HIP, "astraea_probe_kernel_ms: hipEventSynchronize failed");
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, t.ev[index][0], t.ev[index][1]) != hipSuccess)
        return fail(ASTRAEA_ERR_HIP, "astraea_probe_kernel_ms: hipEventElapsedTime failed");
    *ms_out = (double)ms;
    return ASTRAEA_OK;
}

extern "C" int32_t astraea_probe_kernel_count(void) { return astraea::g_timer.count; }
