// Device-ceiling probes behind relax_probe_stream_read / relax_probe_mfma: what a plain streaming read and a bare
// loop of matrix-core instructions reach on the device at hand, for the roofline figures of the benchmark (the
// published peaks are 8 TB/s and 2.5 PFLOP/s; a kernel cannot beat what these reach).  Not part of the hot path.
#include "relax_common.h"

namespace relax {

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// one workgroup of 512 threads per CU reads its own contiguous slice of the buffer, eight independent 16-byte loads per
// lane in flight (64 KB per CU): the access pattern of the weight-streaming kernels without their arithmetic
__global__ __launch_bounds__(512) void stream_read_kernel(const u32x4_t *__restrict__ buf, size_t packets, uint32_t *sink)
{
    constexpr int T = 512, PF = 8;
    const size_t per = (packets + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * per, end = begin + per < packets ? begin + per : packets;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    if (begin < end) {
        const u32x4_t *base = buf + begin;
        const size_t n = end - begin;
        u32x4_t pre[PF];
#pragma unroll
        for (int p = 0; p < PF; ++p) pre[p] = base[min((size_t)threadIdx.x + (size_t)p * T, n - 1)];
        for (size_t at = threadIdx.x; at < n; at += (size_t)PF * T) {
            u32x4_t cur[PF];
#pragma unroll
            for (int p = 0; p < PF; ++p) cur[p] = pre[p];
            if (at + (size_t)PF * T < n) {
#pragma unroll
                for (int p = 0; p < PF; ++p) pre[p] = base[min(at + (size_t)(PF + p) * T, n - 1)];
            }
#pragma unroll
            for (int p = 0; p < PF; ++p)
                if (at + (size_t)p * T < n) acc ^= cur[p];
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = 1u;      // keeps the loads alive; practically never true
}

// 16 independent 32x32x16 fp16 MFMAs per iteration and wavefront (a 128 x 128 accumulator tile), operands in registers
template <int RANDOM>
__global__ __launch_bounds__(256) void mfma_rate_kernel(float *sink, int iters)
{
    const int lane = threadIdx.x & 63;
    half8_t a[4], b[4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t hsh = (uint32_t)(lane * 131 + f * 17 + e + blockIdx.x * 7919) * 2654435761u;
            a[f][e] = (_Float16)(RANDOM ? ((int)((hsh >> 8) & 0xFFFF) - 32768) / 16384.0f : 0.001f * (lane + f + e));
            b[f][e] = (_Float16)(RANDOM ? ((int)((hsh >> 12) & 0xFFFF) - 32768) / 16384.0f : 0.002f * (lane + e));
        }
    float16_t acc[4][4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[f][j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int f = 0; f < 4; ++f) acc[f][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[f], b[j], acc[f][j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[f][j][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_probe_stream_read(const void *buf, size_t bytes, uint32_t *sink, int n_cus, hipStream_t stream)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_cus), dim3(512), 0, stream, (const u32x4_t *)buf, bytes / 16, sink);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(float *sink, int iters, int random_data, int n_cus, hipStream_t stream)
{
    if (random_data) hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(n_cus), dim3(256), 0, stream, sink, iters);
    else hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(n_cus), dim3(256), 0, stream, sink, iters);
    return hipGetLastError();
}

}  // namespace relax
