// Dynamic symmetric INT8 quantizer in front of the attention path (Sec. 2.1, Eq. quant) for gfx950:
//   s_X = max|X| / 127 per tensor (or per head index, Sec. 3.3),  X_hat = clamp(round(X / s_X), -127, 127).
// fp32, fp16 or bf16 in, INT8 and the fp32 scales (device memory) out.  Two passes over the input,
// both bound by HBM: (1) max|X| per group, one 16-byte load per lane and step, reduced per wave
// and per workgroup, one atomic max per workgroup (the bits of a non-negative float order like
// an unsigned integer); (2) one IEEE fp32 division per element, nearest integer with ties to even
// (v_rndne_f32), eight INT8 results per 8-byte store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int QNT = 256;   // threads per workgroup
constexpr int QITEMS = 4;  // 8-element items per thread

// eight consecutive elements of a row as fp32 (widening fp16 / bf16 is exact)
template <int DTYPE>
__device__ __forceinline__ void load8(const uint8_t *p, float (&x)[8])
{
    if (DTYPE == 0) {
        const float4 a = *(const float4 *)p, b = *(const float4 *)(p + 16);
        x[0] = a.x, x[1] = a.y, x[2] = a.z, x[3] = a.w, x[4] = b.x, x[5] = b.y, x[6] = b.z, x[7] = b.w;
    } else {
        const uint4 r = *(const uint4 *)p;
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DTYPE == 1) {
                x[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xffffu));
                x[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
            } else {
                x[2 * i] = __uint_as_float(w[i] << 16);
                x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        }
    }
}

// blockIdx.y = b * H + h; blockIdx.x walks the (L * d / 8) items of that slice.
template <int DTYPE>
__global__ __launch_bounds__(QNT) void absmax_kernel(const QuantParams p)
{
    constexpr int ES = DTYPE == 0 ? 4 : 2;
    __shared__ float wmax[QNT / 64];
    const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H;
    const uint8_t *src = (const uint8_t *)p.src + (int64_t)b * p.ss[0] + (int64_t)h * p.ss[1];
    const int ipr = p.d / 8; // items per row
    const int64_t items = (int64_t)p.L * ipr;
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < QITEMS; ++j) {
        const int64_t it = ((int64_t)blockIdx.x * QITEMS + j) * QNT + threadIdx.x;
        if (it < items) {
            const int64_t row = it / ipr;
            const int c = (int)(it % ipr);
            float x[8];
            load8<DTYPE>(src + row * p.ss[2] + (int64_t)c * 8 * ES, x);
#pragma unroll
            for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < QNT / 64; ++w) m = fmaxf(m, wmax[w]);
        atomicMax(p.amax_bits + (p.per_head ? h : 0), __float_as_uint(m));
    }
}

template <int DTYPE>
__global__ __launch_bounds__(QNT) void quantize_kernel(const QuantParams p)
{
    constexpr int ES = DTYPE == 0 ? 4 : 2;
    const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H;
    const int g = p.per_head ? h : 0;
    const float amax = fmaxf(__uint_as_float(p.amax_bits[g]), 1e-12f);
    const float s = amax / 127.0f; // one IEEE fp32 division
    if (blockIdx.x == 0 && threadIdx.x == 0 && b == 0 && (p.per_head || h == 0)) p.scales[g] = s;
    const uint8_t *src = (const uint8_t *)p.src + (int64_t)b * p.ss[0] + (int64_t)h * p.ss[1];
    int8_t *dst = p.dst + (int64_t)b * p.ds[0] + (int64_t)h * p.ds[1];
    const int ipr = p.d / 8;
    const int64_t items = (int64_t)p.L * ipr;
#pragma unroll
    for (int j = 0; j < QITEMS; ++j) {
        const int64_t it = ((int64_t)blockIdx.x * QITEMS + j) * QNT + threadIdx.x;
        if (it < items) {
            const int64_t row = it / ipr;
            const int c = (int)(it % ipr);
            float x[8];
            load8<DTYPE>(src + row * p.ss[2] + (int64_t)c * 8 * ES, x);
            uint32_t w[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float r = __builtin_rintf(x[i] / s); // IEEE division; nearest integer, ties to even
                r = fminf(fmaxf(r, -127.0f), 127.0f);
                w[i / 4] |= ((uint32_t)(int)r & 0xffu) << (8 * (i % 4));
            }
            *(uint2 *)(dst + row * p.ds[2] + (int64_t)c * 8) = make_uint2(w[0], w[1]);
        }
    }
}

__global__ void zero_amax_kernel(uint32_t *a, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) a[i] = 0u;
}

template <int DTYPE>
int launch_dtype(const QuantParams &p, hipStream_t st)
{
    const int64_t items = (int64_t)p.L * (p.d / 8);
    const dim3 grid((unsigned)((items + QNT * QITEMS - 1) / (QNT * QITEMS)), (unsigned)(p.B * p.H)), block(QNT);
    hipLaunchKernelGGL(absmax_kernel<DTYPE>, grid, block, 0, st, p);
    hipLaunchKernelGGL(quantize_kernel<DTYPE>, grid, block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

int launch_quantize(const QuantParams &p, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int groups = p.per_head ? p.H : 1;
    // cleared by a kernel, not a memset node, so that the call can be captured into a graph
    hipLaunchKernelGGL(zero_amax_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, p.amax_bits, groups);
    if (p.dtype == 0) return launch_dtype<0>(p, st);
    if (p.dtype == 1) return launch_dtype<1>(p, st);
    if (p.dtype == 2) return launch_dtype<2>(p, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
