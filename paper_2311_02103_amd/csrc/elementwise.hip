// Stand-alone forms of the light steps of the layer (RMSNorm, rotary embedding + KV append),
// the rotary table builder and the two dense decode exports used by the bit-exactness tests.
// Inside relax_decoder_layer's decode path these steps run as prologue / epilogue of the
// matrix-vector kernel instead (operator fusion of Sec. 4.2: RMSNorm and element-wise steps
// fold into their neighbours); the kernels here serve the exported calls and the large-n path.
#include "relax_common.h"

namespace relax {

// y[i,:] = x[i,:] * rsqrt(mean(x[i,:]^2) + eps) * w ; one workgroup per row, fp32 reduction.
// The row is read once, eight elements per thread and pass (16-byte loads for fp16, 2 x 16 bytes for fp32), and
// stays in registers between the reduction and the scaling (up to kNormPasses * 2048 columns; longer rows re-read).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
constexpr int kNormPasses = 4;

__device__ inline void load8(const uint16_t *p, float *v)
{
    const u32x4_t raw = *(const u32x4_t *)p;
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) v[2 * j] = h2f((uint16_t)(w[j] & 0xFFFFu)), v[2 * j + 1] = h2f((uint16_t)(w[j] >> 16));
}
__device__ inline void load8(const float *p, float *v)
{
    const float4_t a = *(const float4_t *)p, b = *(const float4_t *)(p + 4);
    v[0] = a.x, v[1] = a.y, v[2] = a.z, v[3] = a.w, v[4] = b.x, v[5] = b.y, v[6] = b.z, v[7] = b.w;
}

template <typename T>
__global__ __launch_bounds__(1024) void rmsnorm_kernel(const T *x, const uint16_t *w, uint16_t *y, int H, float eps)
{
    __shared__ float red[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NT = blockDim.x;
    const size_t base = (size_t)blockIdx.x * H;
    const bool vec = (H & 7) == 0 && H <= kNormPasses * 2048 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) |
                                                                  reinterpret_cast<uintptr_t>(w)) & 15) == 0;
    float v[kNormPasses][8];
    float ss = 0.0f;
    if (vec) {
#pragma unroll
        for (int p = 0; p < kNormPasses; ++p) {
            const int c = (p * NT + tid) * 8;
            if (c < H) {
                load8(x + base + c, v[p]);
#pragma unroll
                for (int e = 0; e < 8; ++e) ss += v[p][e] * v[p][e];
            }
        }
    } else {
        for (int c = tid; c < H; c += NT) {
            float t;
            if (sizeof(T) == 2) t = h2f(((const uint16_t *)x)[base + c]);
            else t = ((const float *)x)[base + c];
            ss += t * t;
        }
    }
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    const float inv = rms_scale(block_total(red, NT >> 6), 1.0f / (float)H, eps);
    if (vec) {
#pragma unroll
        for (int p = 0; p < kNormPasses; ++p) {
            const int c = (p * NT + tid) * 8;
            if (c < H) {
                float wv[8];
                load8(w + c, wv);
                uint32_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = f2h(v[p][2 * j] * inv * wv[2 * j]) | ((uint32_t)f2h(v[p][2 * j + 1] * inv * wv[2 * j + 1]) << 16);
                *(u32x4_t *)(y + base + c) = u32x4_t{o[0], o[1], o[2], o[3]};
            }
        }
    } else {
        for (int c = tid; c < H; c += NT) {
            float t;
            if (sizeof(T) == 2) t = h2f(((const uint16_t *)x)[base + c]);
            else t = ((const float *)x)[base + c];
            y[base + c] = f2h(t * inv * h2f(w[c]));
        }
    }
}

hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int n, int H, float eps, hipStream_t stream)
{
    hipLaunchKernelGGL(rmsnorm_kernel<uint16_t>, dim3(n), dim3(norm_block_threads(H, n)), 0, stream, x, w, y, H, eps);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_f32(const float *x, const uint16_t *w, uint16_t *y, int n, int H, float eps, hipStream_t stream)
{
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(n), dim3(norm_block_threads(H, n)), 0, stream, x, w, y, H, eps);
    return hipGetLastError();
}

// ---- the element-wise steps of a layer as launches of their own ------------------------------------------------------
// For the layer on 3-bit weights (Sec. 5.3 of the paper deploys 3-bit models), whose matmuls have the plain fp16
// epilogue only: residual adds and SwiGLU run between them.  Eight elements per thread, 16-byte accesses; the counts
// are multiples of 8 (hidden and ffn are).
//   x1[i] = x[i] + o[i]                      fp16, fp16 -> fp32   (the residual stream stays fp32 inside a layer)
__global__ __launch_bounds__(256) void add_rows_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ o, float *__restrict__ x1, size_t count8)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= count8) return;
    float a[8], b[8];
    load8(x + t * 8, a), load8(o + t * 8, b);
    *(float4_t *)(x1 + t * 8) = float4_t{a[0] + b[0], a[1] + b[1], a[2] + b[2], a[3] + b[3]};
    *(float4_t *)(x1 + t * 8 + 4) = float4_t{a[4] + b[4], a[5] + b[5], a[6] + b[6], a[7] + b[7]};
}
//   out[i] = fp16(x1[i] + d[i])              fp32, fp16 -> fp16
__global__ __launch_bounds__(256) void add_out_kernel(const float *__restrict__ x1, const uint16_t *__restrict__ d, uint16_t *__restrict__ out, size_t count8)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= count8) return;
    float a[8], b[8];
    load8(x1 + t * 8, a), load8(d + t * 8, b);
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = (uint32_t)f2h(a[2 * j] + b[2 * j]) | ((uint32_t)f2h(a[2 * j + 1] + b[2 * j + 1]) << 16);
    *(u32x4_t *)(out + t * 8) = u32x4_t{w[0], w[1], w[2], w[3]};
}
//   act[i,f] = fp16(silu(gu[i,f]) * gu[i,F+f])    gu [n,2F] fp16 -> act [n,F] fp16
__global__ __launch_bounds__(256) void swiglu_rows_kernel(const uint16_t *__restrict__ gu, uint16_t *__restrict__ act, int F)
{
    const int i = blockIdx.y, f = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (f >= F) return;
    float g[8], u[8];
    load8(gu + (size_t)i * 2 * F + f, g), load8(gu + (size_t)i * 2 * F + F + f, u);
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float a = g[2 * j] / (1.0f + expf(-g[2 * j])) * u[2 * j], b = g[2 * j + 1] / (1.0f + expf(-g[2 * j + 1])) * u[2 * j + 1];
        w[j] = (uint32_t)f2h(a) | ((uint32_t)f2h(b) << 16);
    }
    *(u32x4_t *)(act + (size_t)i * F + f) = u32x4_t{w[0], w[1], w[2], w[3]};
}

hipError_t launch_add_rows(const uint16_t *x, const uint16_t *o, float *x1, size_t count, hipStream_t stream)
{
    const size_t c8 = count / 8;
    hipLaunchKernelGGL(add_rows_kernel, dim3((unsigned)((c8 + 255) / 256)), dim3(256), 0, stream, x, o, x1, c8);
    return hipGetLastError();
}
hipError_t launch_add_out(const float *x1, const uint16_t *d, uint16_t *out, size_t count, hipStream_t stream)
{
    const size_t c8 = count / 8;
    hipLaunchKernelGGL(add_out_kernel, dim3((unsigned)((c8 + 255) / 256)), dim3(256), 0, stream, x1, d, out, c8);
    return hipGetLastError();
}
hipError_t launch_swiglu_rows(const uint16_t *gu, uint16_t *act, int n, int F, hipStream_t stream)
{
    hipLaunchKernelGGL(swiglu_rows_kernel, dim3((unsigned)((F / 8 + 255) / 256), (unsigned)n), dim3(256), 0, stream, gu, act, F);
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
// cache at each row's position.  One workgroup per (row, slice of the heads); a thread owns eight
// consecutive rotation pairs of one head (16-byte loads and stores), or eight v elements.
__global__ __launch_bounds__(256) void rope_append_kernel(uint16_t *qkv, uint16_t *kc, uint16_t *vc, const float *rope, int h,
                                                          int g, int d, int cap, SeqTable st)
{
    const int i = blockIdx.x;
    const RowInfo ri = row_info(st, i);
    const int hd2 = d >> 1, width = (h + 2 * g) * d, per_head = hd2 >> 3;
    uint16_t *row = qkv + (size_t)i * width;
    const size_t tok = ((size_t)ri.slot * cap + ri.pos) * (size_t)(g * d);
    const int items = (h + g) * per_head;                      // d % 16 == 0 for the supported head dims (64, 128)
    for (int u = blockIdx.y * 256 + threadIdx.x; u < items; u += gridDim.y * 256) {
        const int j = u / per_head, t0 = (u - j * per_head) * 8;
        float a[8], b[8];
        load8(row + j * d + t0, a);
        load8(row + j * d + t0 + hd2, b);
        const float *cs = rope + ((size_t)ri.pos * hd2 + t0) * 2;
        uint32_t oa[4], ob[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float4_t c2 = *(const float4_t *)(cs + e * 2);          // cos, sin of t0 + e and t0 + e + 1
            oa[e >> 1] = f2h(a[e] * c2.x - b[e] * c2.y) | ((uint32_t)f2h(a[e + 1] * c2.z - b[e + 1] * c2.w) << 16);
            ob[e >> 1] = f2h(a[e] * c2.y + b[e] * c2.x) | ((uint32_t)f2h(a[e + 1] * c2.w + b[e + 1] * c2.z) << 16);
        }
        const u32x4_t va = {oa[0], oa[1], oa[2], oa[3]}, vb = {ob[0], ob[1], ob[2], ob[3]};
        *(u32x4_t *)(row + j * d + t0) = va;
        *(u32x4_t *)(row + j * d + t0 + hd2) = vb;
        if (j >= h) {
            *(u32x4_t *)(kc + tok + (size_t)(j - h) * d + t0) = va;
            *(u32x4_t *)(kc + tok + (size_t)(j - h) * d + t0 + hd2) = vb;
        }
    }
    const uint16_t *vrow = row + (size_t)(h + g) * d;
    for (int e = (blockIdx.y * 256 + threadIdx.x) * 8; e < g * d; e += gridDim.y * 256 * 8)
        *(u32x4_t *)(vc + tok + e) = *(const u32x4_t *)(vrow + e);
}

hipError_t launch_rope_append(uint16_t *qkv, const relax_layer_dims &dm, const relax_kv_cache &cache, const SeqTable &st,
                              hipStream_t stream)
{
    if (((reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(cache.k) | reinterpret_cast<uintptr_t>(cache.v) |
          reinterpret_cast<uintptr_t>(cache.rope)) & 15) != 0 || dm.head_dim % 16 != 0)
        return hipErrorInvalidValue;                           // the kernel moves 16-byte packets
    const int items = (dm.n_heads + dm.n_kv_heads) * (dm.head_dim / 16);
    const int slices = st.n >= 256 ? 1 : (items + 255) / 256;    // few rows: spread a row's heads over several workgroups
    hipLaunchKernelGGL(rope_append_kernel, dim3(st.n, slices), dim3(256), 0, stream, qkv, cache.k, cache.v, cache.rope, dm.n_heads,
                       dm.n_kv_heads, dm.head_dim, dm.kv_capacity, st);
    return hipGetLastError();
}

// Dense decode exports: element (r,c) <- word r*(k/8)+c/8, nibble c%8, scale c/group of the row's ceil(k/group) scales.
__global__ void unpack_kernel(const uint32_t *q, int8_t *out, int m, int k)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)m * k) return;
    const int r = (int)(idx / k), c = (int)(idx - (size_t)r * k);
    out[idx] = (int8_t)decode_code(q[(size_t)r * (k >> 3) + (c >> 3)], c & 7);
}

__global__ void dequantize_kernel(const uint32_t *q, const uint16_t *s, float *out, int m, int k, int group)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)m * k) return;
    const int r = (int)(idx / k), c = (int)(idx - (size_t)r * k);
    const int G = (k + group - 1) / group;
    out[idx] = (float)decode_code(q[(size_t)r * (k >> 3) + (c >> 3)], c & 7) * h2f(s[(size_t)r * G + c / group]);
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
    hipLaunchKernelGGL(dequantize_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, w.q, w.s, out, w.m, w.k,
                       kGroup << gshift_of(w.group));
    return hipGetLastError();
}

namespace {

__global__ void ws_clear_kernel(uint32_t *p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

__global__ void table_write_kernel(int32_t *table, TableChunk c)
{
    const int j = threadIdx.x;
    if (j < c.count) {
        const int b = c.first + j;
        table[b] = c.q_start[j];
        table[c.B + b] = c.q_len[j];
        table[2 * (size_t)c.B + b] = c.kv_len[j];
        table[3 * (size_t)c.B + b] = c.slot[j];
    }
}

}  // namespace

hipError_t launch_ws_clear(void *base, size_t bytes, hipStream_t stream)
{
    hipLaunchKernelGGL(ws_clear_kernel, dim3(1), dim3(64), 0, stream, (uint32_t *)base, bytes / sizeof(uint32_t));
    return hipGetLastError();
}

hipError_t launch_table_write(int32_t *table, const TableChunk &chunk, hipStream_t stream)
{
    hipLaunchKernelGGL(table_write_kernel, dim3(1), dim3(kTableChunk), 0, stream, table, chunk);
    return hipGetLastError();
}

}  // namespace relax
