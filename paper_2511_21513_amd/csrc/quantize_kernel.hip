// Dynamic symmetric INT8 quantizer in front of the attention path (Sec. 2.1, Eq. quant) for gfx950:
//   s_X = max|X| / 127 per tensor (or per head index, Sec. 3.3),  X_hat = clamp(round(X / s_X), -127, 127).
// fp32, fp16 or bf16 in, INT8 and the fp32 scales (device memory) out.  Two passes over the input,
// both bound by HBM: (1) max|X| of each workgroup's part of a (b, h) slice, 16-byte loads, reduced
// per wave and per workgroup and stored (no atomics: two thousand updates of one word cost more
// than reading the tensor); (2) every workgroup reduces the partial maxima of its group, then one
// IEEE fp32 division per element (done as a multiplication where that provably rounds alike, see quantize8),
// nearest integer with ties to even (v_rndne_f32), eight INT8 results per 8-byte store.  Up to four tensors (Q, K, V) share the two launches: a flat grid whose
// workgroups find their tensor from cumulative counts.  The second pass walks the grid backwards, so
// that it starts in what the first pass left in the caches.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int QNT = 256;   // threads per workgroup
constexpr int QITEMS = 4;  // 8-element items per thread in flight
constexpr int QLOOP = 4;   // rounds of QITEMS items per thread in the second pass: the reduction of the partial
                           // maxima at the start of a workgroup is paid once per 64 KiB of input

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

// Eight elements to INT8: q = clamp(rint(x / s), -127, 127) with x / s the IEEE fp32 quotient and rint to nearest,
// ties to even -- two words of four bytes.  The division is replaced by a multiplication wherever that provably gives
// the same integer: with r = fl(1 / s) (one IEEE division per group) and t = fl(x r), t differs from fl(x / s) by at
// most |x / s| * 3 * 2^-24 (1 + 2^-23) < 2.3e-5 (|x / s| <= 127.5: x is an element of the group whose maximum defines
// s), so whenever t is farther than 2^-14 from every half-integer, t and fl(x / s) lie strictly between the same two
// half-integers and round to the same integer.  Items with an element closer than that (about 1 in 25 for random data)
// take the division itself; the branch is per item of eight elements.
__device__ __forceinline__ void quantize8(const float (&x)[8], float s, float r, uint32_t (&w)[2])
{
    float t[8];
    bool near = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        t[i] = x[i] * r;
        const float f = t[i] - __builtin_floorf(t[i]); // in [0, 1]
        near |= __builtin_fabsf(f - 0.5f) < 6.103515625e-05f;
    }
    if (near) {
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = x[i] / s; // IEEE division
    }
    w[0] = w[1] = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float q = __builtin_rintf(t[i]); // nearest integer, ties to even
        q = fminf(fmaxf(q, -127.0f), 127.0f);
        w[i / 4] |= ((uint32_t)(int)q & 0xffu) << (8 * (i % 4));
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

// Tensor and position of a workgroup in the flat grid of a batch: workgroups [first[i], first[i + 1])
// belong to tensor i and are numbered x-fastest inside it.
struct BatchSlot {
    int ti;
    uint32_t bx, by;
};
__device__ __forceinline__ BatchSlot batch_slot(const QuantBatch &qb, uint32_t lin, const uint32_t (&gx)[4])
{
    int ti = 0;
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (i < qb.n && lin >= qb.first[i]) ti = i;
    const uint32_t rel = lin - qb.first[ti];
    return BatchSlot{ti, rel % gx[ti], rel / gx[ti]};
}

// by = b * H + h; bx walks the (L * d / 8) items of that slice.
template <int DTYPE>
__device__ __forceinline__ void absmax_body(const QuantParams &p, uint32_t bx, uint32_t gdx, uint32_t by)
{
    constexpr int ES = DTYPE == 0 ? 4 : 2;
    __shared__ float wmax[QNT / 64];
    const int bh = (int)by, b = bh / p.H, h = bh % p.H;
    const uint8_t *src = (const uint8_t *)p.src + (int64_t)b * p.ss[0] + (int64_t)h * p.ss[1];
    const int ipr = p.d / 8; // items per row
    const int64_t items = (int64_t)p.L * ipr;
    float m = 0.0f;
    // grid-stride walk, QITEMS loads in flight per thread
    for (int64_t base = (int64_t)bx * QNT + threadIdx.x; base < items; base += (int64_t)gdx * QNT * QITEMS) {
        float x[QITEMS][8];
#pragma unroll
        for (int j = 0; j < QITEMS; ++j) {
            const int64_t it = base + (int64_t)j * gdx * QNT;
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
        p.partial[(int64_t)bh * gdx + bx] = m;
    }
}

__global__ __launch_bounds__(QNT) void absmax_kernel(const QuantBatch qb)
{
    uint32_t gx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) gx[i] = (uint32_t)qb.t[i].n_partial;
    const BatchSlot sl = batch_slot(qb, blockIdx.x, gx);
    const QuantParams &p = qb.t[sl.ti];
    if (p.dtype == 0) absmax_body<0>(p, sl.bx, gx[sl.ti], sl.by);
    else if (p.dtype == 1) absmax_body<1>(p, sl.bx, gx[sl.ti], sl.by);
    else absmax_body<2>(p, sl.bx, gx[sl.ti], sl.by);
}

template <int DTYPE>
__device__ __forceinline__ void quantize_body(const QuantParams &p, uint32_t bx, uint32_t by)
{
    constexpr int ES = DTYPE == 0 ? 4 : 2;
    const int bh = (int)by, b = bh / p.H, h = bh % p.H;
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
    const float rs = 1.0f / s;     // and its reciprocal, for quantize8
    if (bx == 0 && threadIdx.x == 0 && b == 0 && (p.per_head || h == 0)) p.scales[g] = s;
    const uint8_t *src = (const uint8_t *)p.src + (int64_t)b * p.ss[0] + (int64_t)h * p.ss[1];
    int8_t *dst = p.dst + (int64_t)b * p.ds[0] + (int64_t)h * p.ds[1];
    const int ipr = p.d / 8;
    const int64_t items = (int64_t)p.L * ipr;
    for (int r = 0; r < QLOOP; ++r) {
        // QITEMS loads in flight per thread, then the arithmetic and the stores
        float x[QITEMS][8];
        int64_t dofs[QITEMS];
        bool live[QITEMS];
#pragma unroll
        for (int j = 0; j < QITEMS; ++j) {
            const int64_t it = ((int64_t)(bx * QLOOP + r) * QITEMS + j) * QNT + threadIdx.x;
            live[j] = it < items;
            dofs[j] = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) x[j][i] = 0.0f;
            if (live[j]) {
                int64_t so;
                item_offsets<ES>(p, (uint32_t)it, (uint32_t)ipr, so, dofs[j]);
                load8<DTYPE>(src + so, x[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < QITEMS; ++j) {
            uint32_t w[2];
            quantize8(x[j], s, rs, w);
            if (live[j]) *(uint2 *)(dst + dofs[j]) = make_uint2(w[0], w[1]);
        }
    }
}

__global__ __launch_bounds__(QNT) void quantize_kernel(const QuantBatch qb)
{
    uint32_t gx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) gx[i] = qb.gx[i];
    const BatchSlot sl = batch_slot(qb, qb.first[qb.n] - 1u - blockIdx.x, gx); // backwards through the grid
    const QuantParams &p = qb.t[sl.ti];
    if (p.dtype == 0) quantize_body<0>(p, sl.bx, sl.by);
    else if (p.dtype == 1) quantize_body<1>(p, sl.bx, sl.by);
    else quantize_body<2>(p, sl.bx, sl.by);
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
    const float rs = 1.0f / s;                 // and its reciprocal, for quantize8
    if (t == 0) p.scales[gi] = s;
    for (int it = t; it < items; it += NTHR) {
        const int row = it / ipr, c = it - row * ipr;
        float x[8];
        load8<DTYPE>(src + (int64_t)row * p.ss[2] + (int64_t)c * 8 * ES, x);
        uint32_t w[2];
        quantize8(x, s, rs, w);
        *(uint2 *)(dst + (int64_t)row * p.ds[2] + (int64_t)c * 8) = make_uint2(w[0], w[1]);
    }
}

template <int DTYPE>
int launch_rows(const QuantParams &p, hipStream_t st)
{
    const int64_t groups = (int64_t)p.B * p.H * ((p.L + p.q_block - 1) / p.q_block);
    if ((int64_t)p.q_block * p.d <= 4096)
        hipLaunchKernelGGL((quantize_rows_kernel<DTYPE, 64>), dim3((unsigned)((groups + 3) / 4)), dim3(QNT), 0, st, p);
    else
        hipLaunchKernelGGL((quantize_rows_kernel<DTYPE, QNT>), dim3((unsigned)groups), dim3(QNT), 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// Partial maxima per (b, h) slice: about 1024 workgroups in all (four per compute unit, each with 64
// KiB of loads in flight), never more than the slice has work for.
int quantize_partials_per_slice(int B, int H, int L, int d)
{
    const int64_t items = (int64_t)L * (d / 8);
    const int64_t blocks = (items + QNT * QITEMS - 1) / (QNT * QITEMS);
    const int64_t want = (1024 + (int64_t)B * H - 1) / ((int64_t)B * H);
    return (int)(blocks < want ? blocks : want);
}

// n tensors (1..4), each with per_head 0 or 1 and its own partial buffer, in two launches; or one tensor with
// per_head 2 (a scale per block of rows) in one.
int launch_quantize(const QuantParams *ps, int n, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (n < 1 || n > 4) return (int)hipErrorInvalidValue;
    if (ps[0].per_head == 2) {
        if (n != 1) return (int)hipErrorInvalidValue;
        if (ps[0].dtype == 0) return launch_rows<0>(ps[0], st);
        if (ps[0].dtype == 1) return launch_rows<1>(ps[0], st);
        if (ps[0].dtype == 2) return launch_rows<2>(ps[0], st);
        return (int)hipErrorInvalidValue;
    }
    QuantBatch qb;
    memset(&qb, 0, sizeof(qb));
    qb.n = n;
    uint64_t tot_a = 0, tot_q = 0;
    uint32_t first_a[5] = {0, 0, 0, 0, 0};
    for (int i = 0; i < n; ++i) {
        const QuantParams &p = ps[i];
        if (p.per_head == 2 || p.dtype < 0 || p.dtype > 2) return (int)hipErrorInvalidValue;
        qb.t[i] = p;
        const int64_t items = (int64_t)p.L * (p.d / 8);
        qb.gx[i] = (uint32_t)((items + QNT * QITEMS * QLOOP - 1) / (QNT * QITEMS * QLOOP));
        first_a[i] = (uint32_t)tot_a;
        qb.first[i] = (uint32_t)tot_q;
        tot_a += (uint64_t)p.n_partial * (uint64_t)(p.B * p.H);
        tot_q += (uint64_t)qb.gx[i] * (uint64_t)(p.B * p.H);
        if (tot_a > 0x7fffffffull || tot_q > 0x7fffffffull) return (int)hipErrorInvalidValue;
    }
    for (int i = n; i <= 4; ++i) first_a[i] = (uint32_t)tot_a, qb.first[i] = (uint32_t)tot_q;
    QuantBatch qa = qb; // the reduction pass: each workgroup walks its part of a slice
    for (int i = 0; i <= 4; ++i) qa.first[i] = first_a[i];
    hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)tot_a), dim3(QNT), 0, st, qa);
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)tot_q), dim3(QNT), 0, st, qb);
    return (int)hipGetLastError();
}

} // namespace intattn
