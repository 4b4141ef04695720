// Dynamic symmetric INT8 quantizer in front of the attention path (Sec. 2.1, Eq. quant) for gfx950:
//   s_X = max|X| / 127 per tensor (or per head index, Sec. 3.3),  X_hat = clamp(round(X / s_X), -127, 127).
// fp32, fp16 or bf16 in, INT8 and the fp32 scales (device memory) out.  Two passes over the input,
// both bound by HBM: (1) max|X| of each workgroup's part of a (b, h) slice, 16-byte loads, reduced
// per wave and per workgroup and stored (no atomics: two thousand updates of one word cost more
// than reading the tensor); (2) every workgroup reduces the partial maxima of its group, then one
// IEEE fp32 division per element, nearest integer with ties to even (v_rndne_f32), eight INT8
// results per 8-byte store.
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

// Byte offsets of item `it` (eight elements) inside a (b, h) slice.  Rows that follow each other
// without gaps need no division; the host checked that the item count fits 31 bits.
template <int ES>
__device__ __forceinline__ void item_offsets(const QuantParams &p, uint32_t it, uint32_t ipr, int64_t &so, int64_t &dofs)
{
    if (p.ss[2] == (int64_t)p.d * ES && p.ds[2] == (int64_t)p.d) { // wave-uniform
        so = (int64_t)it * 8 * ES;
        dofs = (int64_t)it * 8;
    } else {
        const uint32_t row = it / ipr, c = it - row * ipr;
        so = (int64_t)row * p.ss[2] + (int64_t)c * 8 * ES;
        dofs = (int64_t)row * p.ds[2] + (int64_t)c * 8;
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
    // grid-stride walk, QITEMS loads in flight per thread
    for (int64_t base = (int64_t)blockIdx.x * QNT + threadIdx.x; base < items; base += (int64_t)gridDim.x * QNT * QITEMS) {
        float x[QITEMS][8];
#pragma unroll
        for (int j = 0; j < QITEMS; ++j) {
            const int64_t it = base + (int64_t)j * gridDim.x * QNT;
#pragma unroll
            for (int i = 0; i < 8; ++i) x[j][i] = 0.0f;
            if (it < items) {
                int64_t so, dofs;
                item_offsets<ES>(p, (uint32_t)it, (uint32_t)ipr, so, dofs);
                load8<DTYPE>(src + so, x[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < QITEMS; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[j][i]));
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < QNT / 64; ++w) m = fmaxf(m, wmax[w]);
        p.partial[(int64_t)bh * gridDim.x + blockIdx.x] = m;
    }
}

template <int DTYPE>
__global__ __launch_bounds__(QNT) void quantize_kernel(const QuantParams p)
{
    constexpr int ES = DTYPE == 0 ? 4 : 2;
    const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H;
    const int g = p.per_head ? h : 0;
    // max|X| of the group from the partial maxima: slices (b', h') with h' = h, or all slices
    __shared__ float wmax[QNT / 64];
    float m = 0.0f;
    if (p.per_head) {
        for (int i = threadIdx.x; i < p.B * p.n_partial; i += QNT)
            m = fmaxf(m, p.partial[((int64_t)(i / p.n_partial) * p.H + h) * p.n_partial + i % p.n_partial]);
    } else {
        for (int i = threadIdx.x; i < p.B * p.H * p.n_partial; i += QNT) m = fmaxf(m, p.partial[i]);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < QNT / 64; ++w) m = fmaxf(m, wmax[w]);
    const float amax = fmaxf(m, 1e-12f);
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
            int64_t so, dofs;
            item_offsets<ES>(p, (uint32_t)it, (uint32_t)ipr, so, dofs);
            float x[8];
            load8<DTYPE>(src + so, x);
            uint32_t w[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float r = __builtin_rintf(x[i] / s); // IEEE division; nearest integer, ties to even
                r = fminf(fmaxf(r, -127.0f), 127.0f);
                w[i / 4] |= ((uint32_t)(int)r & 0xffu) << (8 * (i % 4));
            }
            *(uint2 *)(dst + dofs) = make_uint2(w[0], w[1]);
        }
    }
}

// One scale per block of q_block rows of a (b, h) slice (Sec. 3.3; per token at q_block = 1).  A
// group is small, so one team (a wave, or the workgroup for groups above 4096 elements) takes it
// whole: max|X| over the group, then the same arithmetic as above; the second read of the group
// comes from the caches.
template <int DTYPE, int NTHR>
__global__ __launch_bounds__(QNT) void quantize_rows_kernel(const QuantParams p)
{
    constexpr int ES = DTYPE == 0 ? 4 : 2;
    __shared__ float wmax[QNT / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = NTHR == 64 ? lane : tid;
    const int nblk = (p.L + p.q_block - 1) / p.q_block;
    const int64_t gi = NTHR == 64 ? (int64_t)blockIdx.x * (QNT / 64) + wave : (int64_t)blockIdx.x;
    if (gi >= (int64_t)p.B * p.H * nblk) return; // a whole wave of the four-group layout
    const int blk = (int)(gi % nblk), bh = (int)(gi / nblk), b = bh / p.H, h = bh % p.H;
    const int r0 = blk * p.q_block, r1 = min(p.L, r0 + p.q_block);
    const int ipr = p.d / 8, items = (r1 - r0) * ipr;
    const uint8_t *src = (const uint8_t *)p.src + (int64_t)b * p.ss[0] + (int64_t)h * p.ss[1] + (int64_t)r0 * p.ss[2];
    int8_t *dst = p.dst + (int64_t)b * p.ds[0] + (int64_t)h * p.ds[1] + (int64_t)r0 * p.ds[2];
    float m = 0.0f;
    for (int it = t; it < items; it += NTHR) {
        const int row = it / ipr, c = it - row * ipr;
        float x[8];
        load8<DTYPE>(src + (int64_t)row * p.ss[2] + (int64_t)c * 8 * ES, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (NTHR != 64) {
        if (lane == 0) wmax[wave] = m;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < QNT / 64; ++w) m = fmaxf(m, wmax[w]);
    }
    const float s = fmaxf(m, 1e-12f) / 127.0f; // one IEEE fp32 division
    if (t == 0) p.scales[gi] = s;
    for (int it = t; it < items; it += NTHR) {
        const int row = it / ipr, c = it - row * ipr;
        float x[8];
        load8<DTYPE>(src + (int64_t)row * p.ss[2] + (int64_t)c * 8 * ES, x);
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float r = __builtin_rintf(x[i] / s); // IEEE division; nearest integer, ties to even
            r = fminf(fmaxf(r, -127.0f), 127.0f);
            w[i / 4] |= ((uint32_t)(int)r & 0xffu) << (8 * (i % 4));
        }
        *(uint2 *)(dst + (int64_t)row * p.ds[2] + (int64_t)c * 8) = make_uint2(w[0], w[1]);
    }
}

template <int DTYPE>
int launch_dtype(const QuantParams &p, hipStream_t st)
{
    if (p.per_head == 2) {
        const int64_t groups = (int64_t)p.B * p.H * ((p.L + p.q_block - 1) / p.q_block);
        if ((int64_t)p.q_block * p.d <= 4096)
            hipLaunchKernelGGL((quantize_rows_kernel<DTYPE, 64>), dim3((unsigned)((groups + 3) / 4)), dim3(QNT), 0, st, p);
        else
            hipLaunchKernelGGL((quantize_rows_kernel<DTYPE, QNT>), dim3((unsigned)groups), dim3(QNT), 0, st, p);
        return (int)hipGetLastError();
    }
    const int64_t items = (int64_t)p.L * (p.d / 8);
    const dim3 grid((unsigned)((items + QNT * QITEMS - 1) / (QNT * QITEMS)), (unsigned)(p.B * p.H)), block(QNT);
    const dim3 rgrid((unsigned)p.n_partial, grid.y); // the reduction pass: each workgroup walks its part of a slice
    hipLaunchKernelGGL(absmax_kernel<DTYPE>, rgrid, block, 0, st, p);
    hipLaunchKernelGGL(quantize_kernel<DTYPE>, grid, block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// Partial maxima per (b, h) slice: about 2048 workgroups in all, never more than the slice has
// work for.
int quantize_partials_per_slice(int B, int H, int L, int d)
{
    const int64_t items = (int64_t)L * (d / 8);
    const int64_t blocks = (items + QNT * QITEMS - 1) / (QNT * QITEMS);
    const int64_t want = (2048 + (int64_t)B * H - 1) / ((int64_t)B * H);
    return (int)(blocks < want ? blocks : want);
}

int launch_quantize(const QuantParams &p, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (p.dtype == 0) return launch_dtype<0>(p, st);
    if (p.dtype == 1) return launch_dtype<1>(p, st);
    if (p.dtype == 2) return launch_dtype<2>(p, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
