// Bandwidth probes used by the benchmark: a read-only streaming kernel with nontemporal loads (what fraction of the
// HBM peak a bare 16-byte-per-lane stream reaches on this machine) and a plain copy kernel of
// known size (to calibrate the profiler's FETCH_SIZE / WRITE_SIZE counters).
#include "speckv_device.h"

namespace speckv {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const uint4 *__restrict__ src, size_t nvec,
                                                                   unsigned long long *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * kProbeThreads * kProbeUnroll;
    uint32_t acc = 0;
    for (size_t base = (size_t)blockIdx.x * kProbeThreads * kProbeUnroll; base < nvec; base += stride) {
        uint4 w[kProbeUnroll];
#pragma unroll
        for (int j = 0; j < kProbeUnroll; ++j) {
            const size_t i = base + (size_t)j * kProbeThreads + threadIdx.x;
            if (i < nvec) {
                const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src + i));
                w[j] = make_uint4(v.x, v.y, v.z, v.w);
            } else {
                w[j] = make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < kProbeUnroll; ++j) acc ^= w[j].x ^ w[j].y ^ w[j].z ^ w[j].w;
    }
    // The loads must not be dead code, but 65k same-address atomics would dominate the kernel:
    // store only for one bit pattern of the running xor, which real data practically never has.
    if (acc == 0x9e3779b9u) atomicXor(sink, (unsigned long long)acc);
}

__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(uint4 *__restrict__ dst,
                                                                   const uint4 *__restrict__ src, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * kProbeThreads;
    for (size_t i = (size_t)blockIdx.x * kProbeThreads + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

static unsigned probe_blocks(size_t nvec, int per_block, int cap = 16384)
{
    size_t b = (nvec + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > (size_t)cap) b = cap;
    return (unsigned)b;
}

hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, int max_blocks, hipStream_t stream)
{
    const size_t nvec = bytes / 16;
    return launch(probe_read_kernel, dim3(probe_blocks(nvec, kProbeThreads * kProbeUnroll, max_blocks)), dim3(kProbeThreads), stream, static_cast<const uint4 *>(src), nvec,
                       static_cast<unsigned long long *>(sink));
}

hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t stream)
{
    const size_t nvec = bytes / 16;
    return launch(probe_copy_kernel, dim3(probe_blocks(nvec, kProbeThreads)), dim3(kProbeThreads), stream, static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), nvec);
}

} // namespace speckv
