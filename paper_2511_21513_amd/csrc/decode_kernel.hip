// Few query rows against many keys (one decoded token, a short chunk): the work is reading K and V
// once, so it is split over the KEYS, not over query rows.  All query heads that share a KV head,
// times the query rows, are packed into the (at most 31) rows of one 32-row MFMA operand, and the
// three global reductions of IndexSoftmax (Sec. 3.1-3.2: row max, row sum of E_hat, P_hat.V_hat)
// become three launches over 128-key tiles with small per-tile partial results in between:
//   scores:  A_hat = Q_hat K_hat^T of the tile (Sec. 2.1)        -> raw scores, per-tile row max
//   lookup:  global row max -> clip, index map, LUT_hat           -> table indices, per-tile row sum
//   pv:      global row sum -> P_hat (Eq. uint8-prob), P_hat V_hat -> int32 atomics into the accumulator
//   finish:  requantization of the accumulator to INT8
// Integer sums do not depend on the order of the atomics, so the result is the oracle's bit for bit.
// Probabilities go to the signed MFMA as P - 128; row 31 of the operand is all ones, which yields
// the column sums of V of the tile for the correction 128 * colsum.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;
constexpr int BK = 128; // keys per workgroup: one 32-key sub-tile per wave

// packed row r of a (batch, KV head) group: query head kvh * group + r / L, query row r % L
struct RowOf {
    int hq, i;
};
__device__ __forceinline__ RowOf row_of(const FwdParams &p, int kvh, int r)
{
    RowOf x;
    x.hq = kvh * p.group + r / p.L;
    x.i = r % p.L;
    return x;
}

__device__ __forceinline__ bool key_visible(const FwdParams &p, int key, int i)
{
    return key < p.Lk && (!p.causal || key <= p.row_lo + i);
}

// Stages the 128-key tile `t` of a [Lk, D] matrix into LDS with direct global -> LDS loads; the XOR
// swizzle is applied to the global address, and rows at or past Lk come back as zeros from the
// range check of the buffer descriptor (which ends with the last byte of row Lk - 1).
template <int D, bool IS_V>
__device__ __forceinline__ void stage_tile(const int8_t *base, int64_t stride, int Lk, int t, int8_t *dst, int wave, int lane)
{
    const int key0 = t * BK;
    const int8_t *tb = base + (int64_t)key0 * stride;
    const int64_t rem = (int64_t)(Lk - key0 - 1) * stride + D;
    const uint32_t nrec = rem <= 0 ? 0u : (rem > 0xffffffffll ? 0xffffffffu : (uint32_t)rem);
#if defined(__HIP_DEVICE_COMPILE__) // the host pass has neither the descriptor type nor the builtins
    constexpr int NBLK = BK * D / 1024, JB = NBLK / WAVES, CPR = D / 16, RPB = 1024 / D; // 1 KiB blocks: one wave-wide 16-byte load each
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)tb, 0, (int)nrec, 0x00020000);
#pragma unroll
    for (int j = 0; j < JB; ++j) {
        const int blk = wave + WAVES * j;
        const int key = blk * RPB + lane / CPR, cp = lane % CPR;
        const int sw = IS_V ? swz_v<D>(key) : swz_k<D>(key);
        const int goff = key * (int)stride + ((cp ^ sw) << 4); // the host checked 128 * stride < 2^31
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(dst + blk * 1024), 16, goff, 0, 0, 0);
    }
#else
    (void)tb, (void)nrec, (void)dst, (void)wave, (void)lane, (void)stride;
#endif
}

// The index map of Sec. 3.1 with the scheme named in the head's parameters (chosen on the host,
// or by the derivation kernel for device-resident scales).
__device__ __forceinline__ uint32_t index_any(const HeadParams &hp, int t, uint32_t top)
{
    switch (hp.pad[0]) {
    case IDX_MAD24: return index_map<IDX_MAD24>(t, hp, top);
    case IDX_MULHI24: return index_map<IDX_MULHI24>(t, hp, top);
    case IDX_FP32: return index_map<IDX_FP32>(t, hp, top);
    default: return index_map<IDX_FP64>(t, hp, top);
    }
}

// max (IS_MAX) or sum over all 32-key sub-tiles of the per-tile partials of every packed row:
// red[r] for r < R.  src is [nt32][R].  Ends with a barrier.
template <bool IS_MAX>
__device__ __forceinline__ void reduce_partials(const int32_t *src, int nt32, int R, int32_t (*tmp)[32], int32_t *red, int tid)
{
    const int r = tid & 31, c = tid >> 5; // 8 strided parts of the tile range
    int32_t v = IS_MAX ? INT32_MIN : 0;
    if (r < R)
        for (int j = c; j < nt32; j += NT / 32) {
            const int32_t x = src[(int64_t)j * R + r];
            v = IS_MAX ? max(v, x) : v + x;
        }
    tmp[c][r] = v;
    __syncthreads();
    if (tid < 32) {
        int32_t a = tmp[0][tid];
#pragma unroll
        for (int k = 1; k < NT / 32; ++k) a = IS_MAX ? max(a, tmp[k][tid]) : a + tmp[k][tid];
        red[tid] = a;
    }
    __syncthreads();
}

// grid: x = 128-key tile, y = b * Hkv + kvh
template <int D>
__global__ __launch_bounds__(NT) void decode_scores_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;
    __shared__ __attribute__((aligned(1024))) int8_t Ks[BK * D];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int t = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32;
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    stage_tile<D, false>(Kp, p.ks[2], p.Lk, t, Ks, wave, lane);

    // the accumulator of the last launch starts at zero
    if (t == 0)
        for (int e = tid; e < R * D; e += NT) {
            const RowOf ro = row_of(p, kvh, e / D);
            p.dec_acc[((int64_t)(b * p.Hq + ro.hq) * p.L + ro.i) * D + e % D] = 0;
        }

    // Q fragments: packed row n, bytes [32 kb + 16 h, +16)
    const RowOf ro = row_of(p, kvh, n < R ? n : 0);
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (n < R)
            qf[kb] = *(const v4i *)(p.q + (int64_t)b * p.qs[0] + (int64_t)ro.hq * p.qs[1] + (int64_t)ro.i * p.qs[2] + kb * 32 + h * 16);
    }
    __syncthreads(); // the tile is in LDS (the barrier waits for the loads)

    const int8_t *Ksub = Ks + wave * 32 * D;
    const int sw = swz_k<D>(n);
    v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        const v4i kf = *(const v4i *)(Ksub + n * D + (((2 * kb + h) ^ sw) << 4));
        s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf, qf[kb], s, 0, 0, 0);
    }
    // register i of lane (n, h): packed row n, key key0 + acc_key(i, h)
    const int key0 = t * BK + wave * 32;
    int32_t m = INT32_MIN;
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (key_visible(p, key0 + acc_key(i, h), ro.i)) m = max(m, s[i]);
    m = max(m, __shfl_xor(m, 32));
    if (n < R) {
        const int t32 = t * 4 + wave;
        int32_t *dst = p.dec_scores + ((((int64_t)grp * nt32 + t32) * 2 + h) * R + n) * 16;
#pragma unroll
        for (int g = 0; g < 4; ++g) *(v4i *)(dst + 4 * g) = v4i{s[4 * g], s[4 * g + 1], s[4 * g + 2], s[4 * g + 3]};
        if (h == 0) p.dec_pmax[((int64_t)grp * nt32 + t32) * R + n] = m;
    }
}

// grid as above; no matrix work: scores -> table indices and partial row sums
__global__ __launch_bounds__(NT) void decode_lookup_kernel(const FwdParams p)
{
    __shared__ int32_t tmp[NT / 32][32];
    __shared__ int32_t row_max[32];
    __shared__ uint32_t lut_lds[8];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int t = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32;
    if (tid < 8) lut_lds[tid] = p.lut[tid];
    reduce_partials<true>(p.dec_pmax + (int64_t)grp * nt32 * R, nt32, R, tmp, row_max, tid);
    if (n >= R) return; // after the barriers
    const RowOf ro = row_of(p, kvh, n);
    const HeadParams hp = p.hp_table[ro.hq];
    const int mx = row_max[n];
    if (p.dbg_row_max && t == 0 && wave == 0 && h == 0) p.dbg_row_max[(int64_t)(b * p.Hq + ro.hq) * p.L + ro.i] = mx;
    const int t32 = t * 4 + wave, key0 = t32 * 32;
    const int64_t at = (((int64_t)grp * nt32 + t32) * 2 + h) * R + n;
    const int32_t *src = p.dec_scores + at * 16;
    const uint8_t *lut_b = (const uint8_t *)lut_lds;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    uint32_t sum = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const v4i sc = *(const v4i *)(src + 4 * g);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = 4 * g + j;
            uint32_t idx = 32u; // hidden key: probability 0
            if (key_visible(p, key0 + acc_key(i, h), ro.i)) {
                // Delta = max - score (Sec. 3.1), clipped at c_int (Eq. int_clipping), index map, Eq. gather16
                const int64_t delta = (int64_t)mx - (int64_t)sc[j];
                const int dclip = delta < (int64_t)hp.c_int ? (int)delta : hp.c_int;
                idx = index_any(hp, -dclip, (uint32_t)p.top);
                sum += lut_b[idx];
            }
            w[g] |= idx << (8 * j);
        }
    }
    *(v4i *)(p.dec_idx + at * 4) = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
    sum += __shfl_xor(sum, 32); // both lanes of the pair are here: n < R does not depend on h
    if (h == 0) p.dec_psum[((int64_t)grp * nt32 + t32) * R + n] = (int32_t)sum;
}

template <int D>
__global__ __launch_bounds__(NT) void decode_pv_kernel(const FwdParams p)
{
    constexpr int CB = D / 32;
    __shared__ __attribute__((aligned(1024))) int8_t Vs[BK * D];
    __shared__ int32_t tmp[NT / 32][32];
    __shared__ int32_t row_sum[32];
    __shared__ uint32_t lut_lds[8];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int t = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32;
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];
    stage_tile<D, true>(Vp, p.vs[2], p.Lk, t, Vs, wave, lane);
    if (tid < 8) lut_lds[tid] = p.lut[tid];
    reduce_partials<false>(p.dec_psum + (int64_t)grp * nt32 * R, nt32, R, tmp, row_sum, tid); // its barriers also cover Vs and lut_lds

    // the lane's 16 probabilities as bytes P - 128 (Eq. uint8-prob); row 31 is all ones
    const RowOf ro = row_of(p, kvh, n < R ? n : 0);
    const int t32 = t * 4 + wave;
    v4i pf = {0, 0, 0, 0};
    if (n < R) {
        const uint32_t S = (uint32_t)row_sum[n]; // >= 255: the key of the row maximum is visible
        if (p.dbg_row_sum && t == 0 && wave == 0 && h == 0) p.dbg_row_sum[(int64_t)(b * p.Hq + ro.hq) * p.L + ro.i] = (int32_t)S;
        const v4i iw = *(const v4i *)(p.dec_idx + ((((int64_t)grp * nt32 + t32) * 2 + h) * R + n) * 4);
        const uint8_t *lut_b = (const uint8_t *)lut_lds;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t wq = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t idx = ((uint32_t)iw[g] >> (8 * j)) & 0xffu;
                const uint32_t e = idx < 32u ? lut_b[idx] : 0u;
                const uint32_t pr = (510u * e + S) / (2u * S); // round(255 e / S), exact
                wq |= ((pr ^ 0x80u) & 0xffu) << (8 * j);
            }
            pf[g] = (int)wq;
        }
    } else if (n == 31) {
        pf = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
    }

    // V^T fragments of the wave's 32-key sub-tile with the transposing LDS read
    const int8_t *Vsub = Vs + wave * 32 * D;
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1, jj = tr_i >> 1;
    const int key = 8 * (jj >> 2) + 4 * h + (jj & 3);
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int off = key * D + (((2 * cb + tr_g) ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
        const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off));
        const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off + 16 * D));
        const v4i vf = v4i{x0[0], x0[1], x1[0], x1[1]};
        o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0);
    }
    // register 4g + r of lane (n, h): row n, channel 32 cb + 8 g + 4 h + r; row 31 holds the column sums
    int32_t *acc = p.dec_acc + ((int64_t)(b * p.Hq + ro.hq) * p.L + ro.i) * D;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int32_t cs = __shfl(o[cb][i], 31 + 32 * h);
            if (n < R) atomicAdd(acc + cb * 32 + 8 * (i >> 2) + 4 * h + (i & 3), o[cb][i] + 128 * cs);
        }
}

// one thread per four output channels
template <int D>
__global__ __launch_bounds__(NT) void decode_finish_kernel(const FwdParams p)
{
    constexpr int TPR = D / 4; // threads per row
    const int64_t row = (int64_t)blockIdx.x * (NT / TPR) + threadIdx.x / TPR; // (b * Hq + hq) * L + i
    const int c0 = (threadIdx.x % TPR) * 4;
    if (row >= (int64_t)p.B * p.Hq * p.L) return;
    const int i = (int)(row % p.L), bh = (int)(row / p.L), hq = bh % p.Hq, b = bh / p.Hq;
    const HeadParams hp = p.hp_table[hq];
    const v4i a = *(const v4i *)(p.dec_acc + row * D + c0);
    const int64_t half = 1ll << (hp.rq_shift - 1);
    uint32_t packed = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (p.dbg_acc) p.dbg_acc[row * D + c0 + r] = a[r];
        int64_t v = ((int64_t)a[r] * hp.rq_mult + half) >> hp.rq_shift;
        v = v > 127 ? 127 : (v < -127 ? -127 : v);
        packed |= ((uint32_t)(int)v & 0xffu) << (8 * r);
    }
    *(uint32_t *)(p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)i * p.os[2] + c0) = packed;
}

template <int D>
int launch_d(const FwdParams &p, hipStream_t st)
{
    const dim3 grid((unsigned)(p.dec_nt32 / 4), (unsigned)(p.B * p.Hkv)), block(NT);
    hipLaunchKernelGGL(decode_scores_kernel<D>, grid, block, 0, st, p);
    hipLaunchKernelGGL(decode_lookup_kernel, grid, block, 0, st, p);
    hipLaunchKernelGGL(decode_pv_kernel<D>, grid, block, 0, st, p);
    const int64_t rows = (int64_t)p.B * p.Hq * p.L;
    const int rows_per_block = NT / (D / 4);
    hipLaunchKernelGGL(decode_finish_kernel<D>, dim3((unsigned)((rows + rows_per_block - 1) / rows_per_block)), block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// Packed rows (Hq / Hkv) * L must be at most 31, B * Hkv at most 65535; p.hp_table must hold every
// head's parameters with its index-map scheme in pad[0]; the dec_* workspace pointers must be set.
int launch_decode(const FwdParams &p, int d, void *stream)
{
    if (p.dec_rows < 1 || p.dec_rows > 31 || !p.hp_table || (int64_t)p.B * p.Hkv > 65535) return (int)hipErrorInvalidValue;
    if (d == 64) return launch_d<64>(p, (hipStream_t)stream);
    if (d == 128) return launch_d<128>(p, (hipStream_t)stream);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
