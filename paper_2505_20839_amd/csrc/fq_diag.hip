// Measurement aid: a kernel that only reads a buffer.  bench.py times it on the packed weights of the
// decode workload to report which share of the plain streaming-read rate the small-M GEMM reaches.
#include "fq_common.h"
#include "fq_kernels.h"

namespace {

// One workgroup of 512 threads per compute unit; grid-stride 16-byte non-temporal loads, sixteen in
// flight per lane, folded with XOR; one word per workgroup leaves.  (Of the launch shapes tried, this
// one streams 29 MB fastest: 5.7 us against 6.0 - 6.7 us.)
__global__ __launch_bounds__(512) void fq_stream_read_kernel(const fq_v4i* __restrict__ src, size_t chunks,
                                                             unsigned* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 512;
    fq_v4i a = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * 512 + threadIdx.x; i < chunks; i += 16 * stride) {
        fq_v4i v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {                    // sixteen requests in flight, those past the end masked out
            const size_t k = i + j * stride;
            v[j] = k < chunks ? __builtin_nontemporal_load(src + k) : (fq_v4i){0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) a ^= v[j];
    }
    unsigned x = (unsigned)(a[0] ^ a[1] ^ a[2] ^ a[3]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o, 64);
    __shared__ unsigned part[8];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3] ^ part[4] ^ part[5] ^ part[6] ^ part[7];
}

}  // namespace

unsigned fq_stream_read_blocks() { return (unsigned)fq_device_cus(); }

void fq_launch_stream_read(const void* src, size_t bytes, unsigned* sink, hipStream_t stream) {
    hipLaunchKernelGGL(fq_stream_read_kernel, dim3(fq_stream_read_blocks()), dim3(512), 0, stream,
                       static_cast<const fq_v4i*>(src), bytes / 16, sink);
}
