// A plain read-only streaming kernel: what the memory system delivers to 16-byte loads when
// nothing else happens.  The benchmark times it over a buffer as large as a decode launch's
// algorithmic bytes, as the measured ceiling next to the published HBM peak.
#include "tadakv_internal.h"

namespace tadakv {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// A workgroup reads one contiguous run of 64 KiB with 16-byte loads, four per thread in flight, and
// folds what it reads into one word; the word is stored only if it equals a value that does not
// occur, so that the loads cannot be dropped and nothing is written.  Many short workgroups, handed
// out by the hardware as slots free up, reached 6.0 - 6.2 TB/s on 0.45 - 1.2 GB; one resident round of
// workgroups striding through the buffer (the shape of the decode kernels) 5.0 - 5.7 TB/s.
constexpr int kRunPieces = 4096; // 16-byte pieces per workgroup
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *buf, long long n16, unsigned long long *sink)
{
    const long long lo = (long long)blockIdx.x * kRunPieces;
    long long hi = lo + kRunPieces;
    hi = hi < n16 ? hi : n16;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    long long i = lo + threadIdx.x;
    for (; i + 3 * 256 < hi; i += 4 * 256) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = buf[i + k * 256];
#pragma unroll
        for (int k = 0; k < 4; k++) acc ^= v[k];
    }
    for (; i < hi; i += 256) acc ^= buf[i];
    const unsigned long long w = ((unsigned long long)(acc.x ^ acc.z) << 32) | (acc.y + acc.w);
    if (w == 0x5bd1e995deadbeefull && sink) *sink = w;
}

} // namespace

hipError_t launch_stream_read(const void *buf, size_t bytes, unsigned long long *sink, hipStream_t s)
{
    const long long n16 = (long long)(bytes / 16);
    const long long grid = (n16 + kRunPieces - 1) / kRunPieces;
    if (grid < 1 || grid > 0x7FFFFFFF) return note_launch(hipErrorInvalidValue);
    (void)hipGetLastError();
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const u32x4 *)buf, n16, sink);
    return note_launch(hipGetLastError());
}

} // namespace tadakv
