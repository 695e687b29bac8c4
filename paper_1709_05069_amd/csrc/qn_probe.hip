// Bandwidth probes: a plain 128-bit grid-stride copy and a read-only sum.
// They move a known number of bytes, so they calibrate hardware byte counters
// and give the streaming ceiling the Gram and apply passes are compared with.
// And a latency probe: one wavefront running a chain of dependent fp64
// multiply-adds, timed inside the kernel by the constant-rate counter; its
// duration follows the shader clock, which is what the one-workgroup eigen
// kernel is bound by.
#include "qn_internal.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int kProbeThreads = 256;

__global__ __launch_bounds__(kProbeThreads) void probe_copy(
    const v4f *__restrict__ src, v4f *__restrict__ dst, int64_t nvec)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kProbeThreads;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kProbeThreads + threadIdx.x;
         i < nvec; i += stride)
        dst[i] = src[i];
}

// The fastest plain read pattern found on MI355X: each block streams one
// contiguous chunk, eight non-temporal 128-bit loads in flight per lane.
__global__ __launch_bounds__(kProbeThreads) void probe_read(
    const v4f *__restrict__ src, int64_t nvec, float *__restrict__ sink)
{
    int64_t chunk = (nvec + gridDim.x - 1) / gridDim.x;
    chunk = (chunk + kProbeThreads - 1) / kProbeThreads * kProbeThreads;
    const int64_t b0 = static_cast<int64_t>(blockIdx.x) * chunk;
    const int64_t b1 = b0 + chunk < nvec ? b0 + chunk : nvec;
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    int64_t i = b0 + threadIdx.x;
    for (; i + 7 * kProbeThreads < b1; i += 8 * kProbeThreads) {
        v4f t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            t[u] = __builtin_nontemporal_load(src + i + u * kProbeThreads);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc += t[u];
    }
    for (; i < b1; i += kProbeThreads)
        acc += __builtin_nontemporal_load(src + i);
    // one store per thread keeps the loads alive; the value is not meaningful
    sink[static_cast<int64_t>(blockIdx.x) * kProbeThreads + threadIdx.x] =
        (acc.x + acc.y) + (acc.z + acc.w);
}

// out[0]: ticks of the constant 100 MHz counter over `links` dependent fp64
// multiply-adds, out[1]: the same interval by the shader's own cycle counter,
// out[2]: the chain's value (keeps it alive).
__global__ __launch_bounds__(64) void probe_chain(int64_t links, double seed,
                                                  unsigned long long *__restrict__ out)
{
    double x = seed + threadIdx.x;
    const double a = 1.0 - 1.0 / 1048576.0, b = 1.0 / 1024.0;
    const unsigned long long w0 = wall_clock64(), c0 = clock64();
#pragma unroll 1
    for (int64_t i = 0; i < links; i += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
            x = fma(x, a, b);
    }
    const unsigned long long w1 = wall_clock64(), c1 = clock64();
    if (threadIdx.x == 0) {
        out[0] = w1 - w0;
        out[1] = c1 - c0;
        out[2] = static_cast<unsigned long long>(__double_as_longlong(x));
    }
}

}  // namespace qn

using namespace qn;

extern "C" {

int qn_probe_copy(const void *src, void *dst, int64_t bytes, qn_stream_t stream)
{
    if (!src || !dst || bytes < 16 || bytes % 16 != 0 ||
        reinterpret_cast<uintptr_t>(src) % 16 != 0 ||
        reinterpret_cast<uintptr_t>(dst) % 16 != 0)
        return QN_EINVAL;
    Device *dev = nullptr;
    const int rc = get_device(&dev);
    if (rc != QN_OK)
        return rc;
    const int64_t nvec = bytes / 16;
    int64_t want = (nvec + kProbeThreads - 1) / kProbeThreads;
    const int64_t cap = static_cast<int64_t>(dev->cu_count) * 8;
    const int grid = static_cast<int>(want < cap ? want : cap);
    hipLaunchKernelGGL(probe_copy, dim3(grid), dim3(kProbeThreads), 0,
                       static_cast<hipStream_t>(stream),
                       static_cast<const v4f *>(src), static_cast<v4f *>(dst), nvec);
    return check_launch();
}

int qn_probe_read(const void *src, int64_t bytes, float *sink, qn_stream_t stream)
{
    if (!src || !sink || bytes < 16 || bytes % 16 != 0 ||
        reinterpret_cast<uintptr_t>(src) % 16 != 0)
        return QN_EINVAL;
    Device *dev = nullptr;
    const int rc = get_device(&dev);
    if (rc != QN_OK)
        return rc;
    const int64_t nvec = bytes / 16;
    const int grid = dev->cu_count * 2;   // sink holds qn_probe_sink_floats() >= grid*256 floats
    hipLaunchKernelGGL(probe_read, dim3(grid), dim3(kProbeThreads), 0,
                       static_cast<hipStream_t>(stream),
                       static_cast<const v4f *>(src), nvec, sink);
    return check_launch();
}

int qn_probe_chain(int64_t links, unsigned long long *out, qn_stream_t stream)
{
    if (!out || links < 8 || links % 8 != 0 || links > (static_cast<int64_t>(1) << 30))
        return QN_EINVAL;
    Device *dev = nullptr;
    const int rc = get_device(&dev);
    if (rc != QN_OK)
        return rc;
    hipLaunchKernelGGL(probe_chain, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       links, 0.5, out);
    return check_launch();
}

int qn_probe_sink_floats(void)
{
    Device *dev = nullptr;
    if (get_device(&dev) != QN_OK)
        return -1;
    return dev->cu_count * 8 * kProbeThreads;
}

}  // extern "C"
