// Stand-alone forms of the light steps of the layer (RMSNorm, rotary embedding + KV append),
// the rotary table builder and the two dense decode exports used by the bit-exactness tests.
// Inside relax_decoder_layer's decode path these steps run as prologue / epilogue of the
// matrix-vector kernel instead (operator fusion of Sec. 4.2: RMSNorm and element-wise steps
// fold into their neighbours); the kernels here serve the exported calls and the large-n path.
#include "relax_common.h"

namespace relax {

// y[i,:] = x[i,:] * rsqrt(mean(x[i,:]^2) + eps) * w ; one workgroup per row, fp32 reduction.
template <typename T>
__device__ inline float load_as_float(const T *p, size_t i);
template <>
__device__ inline float load_as_float<uint16_t>(const uint16_t *p, size_t i) { return h2f(p[i]); }
template <>
__device__ inline float load_as_float<float>(const float *p, size_t i) { return p[i]; }

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T *x, const uint16_t *w, uint16_t *y, int H, float eps)
{
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t base = (size_t)blockIdx.x * H;
    float ss = 0.0f;
    for (int c = tid; c < H; c += 256) {
        float v = load_as_float<T>(x, base + c);
        ss += v * v;
    }
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)H + eps);
    for (int c = tid; c < H; c += 256) y[base + c] = f2h(load_as_float<T>(x, base + c) * inv * h2f(w[c]));
}

hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int n, int H, float eps, hipStream_t stream)
{
    hipLaunchKernelGGL(rmsnorm_kernel<uint16_t>, dim3(n), dim3(256), 0, stream, x, w, y, H, eps);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_f32(const float *x, const uint16_t *w, uint16_t *y, int n, int H, float eps, hipStream_t stream)
{
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(n), dim3(256), 0, stream, x, w, y, H, eps);
    return hipGetLastError();
}

// table[pos][t] = (cos, sin)(pos * base^(-2t/d)), everything in fp64 until the final rounding.
__global__ void rope_table_kernel(float *table, int cap, int hd2, int d, double base)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= cap * hd2) return;
    const int pos = idx / hd2, t = idx - pos * hd2;
    const double theta = pow(base, -2.0 * (double)t / (double)d);
    double s, c;
    sincos((double)pos * theta, &s, &c);
    table[2 * (size_t)idx] = (float)c;
    table[2 * (size_t)idx + 1] = (float)s;
}

hipError_t launch_rope_table(const relax_layer_dims &dm, float *table, hipStream_t stream)
{
    const int hd2 = dm.head_dim / 2, total = dm.kv_capacity * hd2;
    hipLaunchKernelGGL(rope_table_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, table, dm.kv_capacity, hd2,
                       dm.head_dim, (double)dm.rope_base);
    return hipGetLastError();
}

// Rotary embedding in place on the q and k columns of qkv, then append k (rotated) and v to the
// cache at each row's position.  One workgroup per row; a thread owns one rotation pair or one
// v element pair.
__global__ __launch_bounds__(256) void rope_append_kernel(uint16_t *qkv, uint16_t *kc, uint16_t *vc, const float *rope, int h,
                                                          int g, int d, int cap, SeqTable st)
{
    const int i = blockIdx.x;
    const RowInfo ri = row_info(st, i);
    const int hd2 = d >> 1, width = (h + 2 * g) * d;
    uint16_t *row = qkv + (size_t)i * width;
    const size_t tok = ((size_t)ri.slot * cap + ri.pos) * (size_t)(g * d);
    const int nqk = (h + g) * hd2;
    for (int u = threadIdx.x; u < nqk; u += blockDim.x) {
        const int j = u / hd2, t = u - j * hd2;
        const float c = rope[((size_t)ri.pos * hd2 + t) * 2], s = rope[((size_t)ri.pos * hd2 + t) * 2 + 1];
        const float a = h2f(row[j * d + t]), b = h2f(row[j * d + t + hd2]);
        const uint16_t oa = f2h(a * c - b * s), ob = f2h(a * s + b * c);
        row[j * d + t] = oa;
        row[j * d + t + hd2] = ob;
        if (j >= h) {
            kc[tok + (size_t)(j - h) * d + t] = oa;
            kc[tok + (size_t)(j - h) * d + t + hd2] = ob;
        }
    }
    const uint16_t *vrow = row + (size_t)(h + g) * d;
    for (int e = threadIdx.x; e < g * d; e += blockDim.x) vc[tok + e] = vrow[e];
}

hipError_t launch_rope_append(uint16_t *qkv, const relax_layer_dims &dm, const relax_kv_cache &cache, const SeqTable &st,
                              hipStream_t stream)
{
    hipLaunchKernelGGL(rope_append_kernel, dim3(st.n), dim3(256), 0, stream, qkv, cache.k, cache.v, cache.rope, dm.n_heads,
                       dm.n_kv_heads, dm.head_dim, dm.kv_capacity, st);
    return hipGetLastError();
}

// Dense decode exports: element (r,c) <- word r*(k/8)+c/8, nibble c%8, scale group c/32.
__global__ void unpack_kernel(const uint32_t *q, int8_t *out, int m, int k)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)m * k) return;
    const int r = (int)(idx / k), c = (int)(idx - (size_t)r * k);
    out[idx] = (int8_t)decode_code(q[(size_t)r * (k >> 3) + (c >> 3)], c & 7);
}

__global__ void dequantize_kernel(const uint32_t *q, const uint16_t *s, float *out, int m, int k)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)m * k) return;
    const int r = (int)(idx / k), c = (int)(idx - (size_t)r * k);
    const int G = (k + kGroup - 1) / kGroup;
    out[idx] = (float)decode_code(q[(size_t)r * (k >> 3) + (c >> 3)], c & 7) * h2f(s[(size_t)r * G + c / kGroup]);
}

hipError_t launch_unpack(const relax_qmat &w, int8_t *out, hipStream_t stream)
{
    const size_t total = (size_t)w.m * w.k;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, w.q, out, w.m, w.k);
    return hipGetLastError();
}

hipError_t launch_dequantize(const relax_qmat &w, float *out, hipStream_t stream)
{
    const size_t total = (size_t)w.m * w.k;
    hipLaunchKernelGGL(dequantize_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, w.q, w.s, out, w.m, w.k);
    return hipGetLastError();
}

}  // namespace relax
