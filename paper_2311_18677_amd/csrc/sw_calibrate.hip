// Measurement support: a plain streaming read of a device buffer, the practical
// ceiling a kernel that must read N bytes from HBM once can be held against
// (the token phase is bound by exactly such a read of the KV cache, paper
// section 3.5).  Every workgroup walks the buffer with a grid stride, 16 bytes
// per lane and eight loads in flight, XORs what it reads and stores one word.
// (Giving every workgroup one contiguous share instead measured slower at the
// sizes of a decode batch.)
#include "sw_internal.h"

namespace {

typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kInFlight = 8;

__global__ __launch_bounds__(kThreads)
void sw_stream_read_kernel(const uint4_t *src, unsigned long long n16, unsigned *sink)
{
    const unsigned long long stride = (unsigned long long)gridDim.x * kThreads;
    unsigned long long i = (unsigned long long)blockIdx.x * kThreads + threadIdx.x;
    uint4_t acc = uint4_t{0u, 0u, 0u, 0u};
    for (; i + (kInFlight - 1) * stride < n16; i += kInFlight * stride) {
        uint4_t x[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) x[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc ^= x[u];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    unsigned r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    // wave, then workgroup
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) r ^= (unsigned)__shfl_xor((int)r, s, 64);
    __shared__ unsigned part[kThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

}  // namespace

hipError_t sw_launch_stream_read(const void *src, unsigned long long n_bytes, unsigned *sink,
                                 int workgroups, hipStream_t stream, const SwLaunchEvents *ev)
{
    return sw_launch(sw_stream_read_kernel, dim3((unsigned)workgroups), dim3(kThreads), 0, stream, ev,
                     reinterpret_cast<const uint4_t *>(src), n_bytes / 16, sink);
}
