// IndexSoftmax as an operator of its own (Sec. 3.1-3.2) on INT32 logits [rows, cols] in device
// memory, UINT8 probabilities out: per row  max -> clip at c_int -> index map -> LUT_hat -> integer
// sum -> P = round(255 E / S).  Bound by HBM: 4 bytes in, 1 byte out per element when the row is
// read once.  A row is handled by a team of 64 lanes (cols <= 2048, four rows per workgroup) or 256
// threads; it stays in registers between the three steps when it fits (cols <= 16384), otherwise
// it is streamed three times (the later passes mostly hit the caches).  The 32 table values and
// the 33 probabilities a row can take live in lanes and are fetched with a lane permute.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

__device__ __forceinline__ int32_t wave_max(int32_t v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = max(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// NTHR threads per row (64: a wave, no barriers; 256: the workgroup).  NCH > 0: the row is held in
// NCH groups of four logits per thread; NCH == 0: streamed.  MODE: IDX_TOP24 (the index is the top
// byte of a 24-bit multiply-add; thresholds up to several thousand) or IDX_FP64 (every threshold).
// Table indices travel as idx * 4, the byte offset the lane permute takes, so that a lookup is one
// permute: LUT_hat[idx] and later P[idx] live in lane idx.
template <int NTHR, int NCH, int MODE>
__global__ __launch_bounds__(256) void index_softmax_kernel(const SoftmaxParams p)
{
    __shared__ int32_t red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = NTHR == 64 ? lane : tid;
    const int64_t row = NTHR == 64 ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    if (row >= p.rows) return; // a whole wave of the four-row layout; the 256-thread layout has no spare rows
    const int cols = p.cols;
    const int n_vis = p.causal ? (int)(row % p.rows_per_matrix) + cols - p.rows_per_matrix + 1 : cols;
    const int32_t *src = (const int32_t *)((const uint8_t *)p.logits + row * p.ls);
    uint8_t *dst = p.prob + row * p.ps;
    const HeadParams hp = p.hp;
    const uint32_t c_int = (uint32_t)hp.c_int, top4 = (uint32_t)p.top * 4u;
    const uint32_t lutv = (p.lut[lane >> 2] >> (8 * (lane & 3))) & 0xffu; // LUT_hat[lane] (0 beyond the table; up to 64 entries)
    const double negr = idx_fp64_factor(hp);
    const int mul = (int)hp.idx_mul;

    auto load4 = [&](int c, int32_t (&x)[4]) __attribute__((always_inline)) {
        if (p.vec_in && c + 3 < cols) {
            const v4i q = *(const v4i *)(src + c);
            x[0] = q[0], x[1] = q[1], x[2] = q[2], x[3] = q[3];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = c + e < cols ? src[c + e] : 0;
        }
    };
    auto team_max = [&](int32_t v) __attribute__((always_inline)) {
        v = wave_max(v);
        if (NTHR == 64) return v;
        if (lane == 0) red[0][wave] = v;
        __syncthreads();
        return max(max(red[0][0], red[0][1]), max(red[0][2], red[0][3]));
    };
    auto team_sum = [&](uint32_t v) __attribute__((always_inline)) {
        v = wave_sum(v);
        if (NTHR == 64) return v;
        if (lane == 0) red[1][wave] = (int32_t)v;
        __syncthreads();
        return (uint32_t)red[1][0] + (uint32_t)red[1][1] + (uint32_t)red[1][2] + (uint32_t)red[1][3];
    };
    // 4 * table index of a visible logit -- Delta = max - A needs 33 bits; as an unsigned difference it is
    // exact, and the clip brings it to at most 2^30
    auto index4 = [&](int32_t x, int32_t m) __attribute__((always_inline)) {
        const uint32_t delta = (uint32_t)m - (uint32_t)x;
        const int tneg = -(int)(delta < c_int ? delta : c_int);
        if (MODE == IDX_TOP24) return (((uint32_t)__mul24(tneg, mul) + hp.idx_add) >> 22) & 0x3fcu;
        return (uint32_t)(int)__builtin_fma((double)tneg, negr, 0.5) << 2;
    };
    // the four indices (times 4) of the group at column c as bytes of one word; a hidden column takes the
    // last table entry, which is 0 by Eq. lut16.  Groups that are visible as a whole skip the selects.
    auto index_word = [&](const int32_t (&x)[4], int32_t m, int c) __attribute__((always_inline)) {
        uint32_t w = 0;
        if (c + 3 < n_vis) {
#pragma unroll
            for (int e = 0; e < 4; ++e) w |= index4(x[e], m) << (8 * e);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) w |= (c + e < n_vis ? index4(x[e], m) : top4) << (8 * e);
        }
        return w;
    };
    // lane value `v` of the lanes named by the four bytes of w (byte offsets idx * 4), summed / packed
    auto gather_sum = [&](uint32_t v, uint32_t w) __attribute__((always_inline)) {
        uint32_t acc = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc += (uint32_t)__builtin_amdgcn_ds_bpermute((int)((w >> (8 * e)) & 0xffu), (int)v);
        return acc;
    };
    auto gather_pack = [&](uint32_t v, uint32_t w) __attribute__((always_inline)) {
        uint32_t packed = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) packed |= (uint32_t)__builtin_amdgcn_ds_bpermute((int)((w >> (8 * e)) & 0xffu), (int)v) << (8 * e);
        return packed;
    };
    auto store4 = [&](int c, uint32_t packed) __attribute__((always_inline)) {
        if (p.vec_out && c + 3 < cols) *(uint32_t *)(dst + c) = packed;
        else
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c + e < cols) dst[c + e] = (uint8_t)(packed >> (8 * e));
    };

    constexpr int NREG = NCH > 0 ? NCH : 1;
    int32_t v[NREG][4];
    int32_t m = INT32_MIN;
    // ---- row max over the visible columns
    if (NCH > 0) {
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int c = (t + NTHR * j) * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[j][e] = 0;
            if (c < cols) load4(c, v[j]);
        }
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int c = (t + NTHR * j) * 4;
            if (c + 3 < n_vis) {
                m = max(max(m, v[j][0]), max(v[j][1], max(v[j][2], v[j][3])));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (c + e < n_vis) m = max(m, v[j][e]);
            }
        }
    } else {
        for (int c = t * 4; c < n_vis; c += NTHR * 4) {
            int32_t x[4];
            load4(c, x);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c + e < n_vis) m = max(m, x[e]);
        }
    }
    m = team_max(m);

    // ---- clip, index map, LUT_hat, row sum; the indices of a resident row are kept as bytes
    uint32_t w[NREG];
    uint32_t sum = 0;
    if (NCH > 0) {
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            w[j] = index_word(v[j], m, (t + NTHR * j) * 4);
            sum += gather_sum(lutv, w[j]);
        }
    } else {
        // every lane takes part in every permute: the trip count is rounded up for the whole team
        for (int c = t * 4; c - t * 4 < n_vis; c += NTHR * 4) {
            int32_t x[4] = {0, 0, 0, 0};
            if (c < n_vis) load4(c, x);
            sum += gather_sum(lutv, index_word(x, m, c));
        }
    }
    const uint32_t S = team_sum(sum); // >= 255: the column of the row maximum is visible

    // ---- Eq. uint8-prob: lane l holds the probability of table index l (0 beyond the table)
    const uint32_t ptv = (510u * lutv + S) / (2u * S);
    if (NCH > 0) {
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int c = (t + NTHR * j) * 4;
            const uint32_t packed = gather_pack(ptv, w[j]);
            if (c < cols) store4(c, packed);
        }
    } else {
        for (int c = t * 4; c - t * 4 < cols; c += NTHR * 4) {
            int32_t x[4] = {0, 0, 0, 0};
            if (c < n_vis) load4(c, x);
            const uint32_t packed = gather_pack(ptv, index_word(x, m, c));
            if (c < cols) store4(c, packed);
        }
    }
}

template <int NTHR, int NCH> int launch_one(const SoftmaxParams &p, hipStream_t st)
{
    const int64_t blocks = NTHR == 64 ? (p.rows + 3) / 4 : p.rows;
    if (p.hp.pad[0] == IDX_TOP24)
        hipLaunchKernelGGL((index_softmax_kernel<NTHR, NCH, IDX_TOP24>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((index_softmax_kernel<NTHR, NCH, IDX_FP64>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// rows <= 2^31 - 1 workgroups' worth, 1 <= cols <= 2^29; strides in bytes; vec_in / vec_out say whether
// every row starts 16-byte (logits) / 4-byte (prob) aligned, which allows the wide accesses; p.hp holds
// c_int and the index-map constants with the scheme in pad[0]: IDX_TOP24 or IDX_FP64.
int launch_index_softmax(const SoftmaxParams &p, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int c = p.cols;
    if (c <= 256) return launch_one<64, 1>(p, st);
    if (c <= 512) return launch_one<64, 2>(p, st);
    if (c <= 1024) return launch_one<64, 4>(p, st);
    if (c <= 2048) return launch_one<64, 8>(p, st);
    if (c <= 4096) return launch_one<256, 4>(p, st);
    if (c <= 8192) return launch_one<256, 8>(p, st);
    if (c <= 16384) return launch_one<256, 16>(p, st);
    return launch_one<256, 0>(p, st);
}

} // namespace intattn
