// Two reference launches for the benchmark: what a launch costs before it does anything,
// and what reading a given number of bytes once costs with the multiply kernel's launch
// geometry.  They bound what any one-launch-per-product kernel can reach on this protocol.
#include "rsr_internal.h"

namespace rsr {
namespace {

// Does nothing; takes the multiply kernel's place in a launch sequence.
__global__ __launch_bounds__(1024) void k_probe_empty() {}

// Every wave reads its share of consecutive 16-byte-per-lane pieces (1 KiB each; shares
// differ by at most one piece, the longer ones first), as the multiply kernel reads its
// slabs: all requests of the wave first (up to MAXP pieces at a time), then one use of the
// data.  The sum is stored only if it has a value it cannot have (the loads must not be
// optimised away).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbePieces = 8;

__global__ __launch_bounds__(1024) void k_probe_read(const u32x4 *__restrict__ src, long long pieces,
                                                     long long per, long long rem,
                                                     uint32_t *__restrict__ sink) {
    const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    const long long first = wave * per + (wave < rem ? wave : rem);
    const long long count = per + (wave < rem ? 1 : 0);
    uint32_t acc = 0;
    for (long long i0 = 0; i0 < count; i0 += kProbePieces) {
        u32x4 q[kProbePieces];
#pragma unroll
        for (int j = 0; j < kProbePieces; ++j)
            if (i0 + j < count) q[j] = __builtin_nontemporal_load(&src[(first + i0 + j) * 64 + lane]);
#pragma unroll
        for (int j = 0; j < kProbePieces; ++j)
            if (i0 + j < count) acc += q[j].x ^ q[j].y ^ q[j].z ^ q[j].w;
    }
    if (acc == 0x9e3779b9u && sink) sink[0] = acc;
}

}  // namespace

hipError_t launch_probe_empty(int workgroups, int threads, int lds_bytes, hipStream_t stream) {
    static std::atomic<size_t> enabled[kMaxDevices];
    int device = 0;
    if (hipError_t e = hipGetDevice(&device)) return e;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(k_probe_empty), (size_t)lds_bytes,
                                          device, enabled))
        return e;
    hipLaunchKernelGGL(k_probe_empty, dim3((unsigned)workgroups), dim3((unsigned)threads), (size_t)lds_bytes,
                       stream);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, int64_t bytes, int workgroups, int threads, void *sink,
                             hipStream_t stream) {
    const long long pieces = bytes / 1024;
    const long long waves = (long long)workgroups * (threads / 64);
    hipLaunchKernelGGL(k_probe_read, dim3((unsigned)workgroups), dim3((unsigned)threads), 0, stream,
                       static_cast<const u32x4 *>(src), pieces, pieces / waves, pieces % waves,
                       static_cast<uint32_t *>(sink));
    return hipGetLastError();
}

}  // namespace rsr
