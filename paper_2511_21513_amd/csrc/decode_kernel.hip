// Few query rows against many keys (one decoded token, a short chunk): the work is reading K and V
// once, so it is split over the KEYS, not over query rows.  All query heads that share a KV head,
// times the query rows, are packed into the (at most 31) rows of one 32-row MFMA operand, and the
// three global reductions of IndexSoftmax (Sec. 3.1-3.2: row max, row sum of E_hat, P_hat.V_hat)
// become three launches over chunks of 128-key tiles with small partial results in between:
//   scores:  A_hat = Q_hat K_hat^T of the tile (Sec. 2.1)        -> raw scores, per-tile row max
//   lookup:  global row max -> clip, index map, LUT_hat           -> table indices, per-tile row sum
//   pv:      global row sum -> P_hat (Eq. uint8-prob), P_hat V_hat -> per-tile partial accumulators
//   finish:  sum of the partial accumulators, requantization to INT8
// Integer sums do not depend on the order of the additions, so the result equals the row-by-row definition bit for bit.
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

// max (IS_MAX) or sum over all 32-key sub-tiles of the per-tile partials of every packed row:
// red[r] for r < R.  src is [nt32][R].  Thread tid takes row tid % R of every (NT / R)-th sub-tile, so
// all threads load (several loads in flight each), then one LDS atomic per thread.  Ends with a barrier.
template <bool IS_MAX>
__device__ __forceinline__ void reduce_partials(const int32_t *src, int nt32, int R, int32_t *red, int tid)
{
    if (tid < 32) red[tid] = IS_MAX ? INT32_MIN : 0;
    __syncthreads();
    const int per = NT / R; // sub-tiles covered per pass
    if (tid < per * R) {
        const int r = tid % R;
        int32_t v = IS_MAX ? INT32_MIN : 0;
#pragma unroll 8
        for (int j = tid / R; j < nt32; j += per) {
            const int32_t x = src[(int64_t)j * R + r];
            v = IS_MAX ? max(v, x) : v + x;
        }
        if (IS_MAX) atomicMax(red + r, v);
        else atomicAdd(red + r, v);
    }
    __syncthreads();
}

// The three kernels below share a grid: x = chunk of p.dec_tpw consecutive 128-key tiles,
// y = b * Hkv + kvh.  Partial row maxima and sums are kept per (chunk, wave): np = 4 * chunks per row.

template <int D>
__global__ __launch_bounds__(NT) void decode_scores_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;
    __shared__ __attribute__((aligned(1024))) int8_t Ks0[BK * D];
    __shared__ __attribute__((aligned(1024))) int8_t Ks1[BK * D];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32, nt = nt32 / 4;
    const int t0 = chunk * p.dec_tpw, t1 = min(t0 + p.dec_tpw, nt);
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    stage_tile<D, false>(Kp, p.ks[2], p.Lk, t0, Ks0, wave, lane);

    // Q fragments: packed row n, bytes [32 kb + 16 h, +16)
    const RowOf ro = row_of(p, kvh, n < R ? n : 0);
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (n < R)
            qf[kb] = *(const v4i *)(p.q + (int64_t)b * p.qs[0] + (int64_t)ro.hq * p.qs[1] + (int64_t)ro.i * p.qs[2] + kb * 32 + h * 16);
    }
    const int sw = swz_k<D>(n);
    int32_t m = INT32_MIN;
    publish_tiles_barrier(); // tile t0 is in LDS
    // One tile: the next one is requested first, into the buffer that was read one step ago (a
    // barrier lies in between).  The buffers are named statically in the loop below, so that the
    // compiler lets the reads of one proceed while loads into the other are in flight.
    auto step = [&](int t, const int8_t *cur, int8_t *nxt) __attribute__((always_inline)) {
        if (t + 1 < t1) stage_tile<D, false>(Kp, p.ks[2], p.Lk, t + 1, nxt, wave, lane);
        const int8_t *Ksub = cur + wave * 32 * D;
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const v4i kf = *(const v4i *)(Ksub + n * D + (((2 * kb + h) ^ sw) << 4));
            s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf, qf[kb], s, 0, 0, 0);
        }
        // register i of lane (n, h): packed row n, key key0 + acc_key(i, h)
        const int t32 = t * 4 + wave, key0 = t32 * 32;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (key_visible(p, key0 + acc_key(i, h), ro.i)) m = max(m, s[i]);
        if (n < R) {
            int32_t *dst = p.dec_scores + ((((int64_t)grp * nt32 + t32) * 2 + h) * R + n) * 16;
#pragma unroll
            for (int g = 0; g < 4; ++g) *(v4i *)(dst + 4 * g) = v4i{s[4 * g], s[4 * g + 1], s[4 * g + 2], s[4 * g + 3]};
        }
        publish_tiles_barrier(); // the next tile has arrived, and every wave is done with this one
    };
    for (int t = t0; t < t1; t += 2) {
        step(t, Ks0, Ks1);
        if (t + 1 < t1) step(t + 1, Ks1, Ks0);
    }
    m = max(m, __shfl_xor(m, 32));
    if (n < R && h == 0) p.dec_pmax[((int64_t)grp * p.dec_np + chunk * 4 + wave) * R + n] = m;
}

// No matrix work: scores -> table indices and partial row sums.  The scores of a chunk are one
// contiguous array ([sub-tile][h][row][16]); every thread takes groups of four of them, whatever
// their row, so that all lanes work although only a few rows of the MFMA operand are in use.
__global__ __launch_bounds__(NT) void decode_lookup_kernel(const FwdParams p)
{
    __shared__ int32_t row_max[32];
    __shared__ int32_t row_i[32];        // query row of packed row r
    __shared__ HeadParams row_hp[32];    // its head's parameters
    __shared__ uint32_t sums[32];
    __shared__ uint32_t lut_lds[16];
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32, nt = nt32 / 4;
    const int t0 = chunk * p.dec_tpw, t1 = min(t0 + p.dec_tpw, nt);
    if (tid < 16) lut_lds[tid] = p.lut[tid];
    if (tid < R) {
        const RowOf ro = row_of(p, kvh, tid);
        row_i[tid] = ro.i;
        row_hp[tid] = p.hp_table[ro.hq];
        sums[tid] = 0;
    }
    reduce_partials<true>(p.dec_pmax + (int64_t)grp * p.dec_np * R, p.dec_np, R, row_max, tid);
    if (p.dbg_row_max && chunk == 0 && tid < R) {
        const RowOf ro = row_of(p, kvh, tid);
        p.dbg_row_max[(int64_t)(b * p.Hq + ro.hq) * p.L + ro.i] = row_max[tid];
    }
    const uint8_t *lut_b = (const uint8_t *)lut_lds;
    // group q of four scores: q = ((sub-tile * 2 + h) * R + n) * 4 + g holds registers 4g .. 4g+3 of lane (n, h)
    const int64_t base = (int64_t)grp * nt32 + (int64_t)t0 * 4; // first sub-tile of the chunk
    const int nq = (t1 - t0) * 4 * 2 * R * 4;
    for (int q = tid; q < nq; q += NT) {
        const int g = q & 3, rn = q >> 2, n = rn % R, sh = rn / R, h = sh & 1, t32l = sh >> 1;
        const int key0 = (t0 * 4 + t32l) * 32;
        const v4i sc = *(const v4i *)(p.dec_scores + (base * 2 * R * 4 + q) * 4);
        const int mx = row_max[n], ri = row_i[n];
        const HeadParams &hp = row_hp[n];
        uint32_t w = 0, sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t idx = 64u; // hidden key: probability 0 (one past the largest table, 2^6 entries)
            if (key_visible(p, key0 + acc_key(4 * g + j, h), ri)) {
                // Delta = max - score (Sec. 3.1), clipped at c_int (Eq. int_clipping), index map, Eq. gather16
                const int64_t delta = (int64_t)mx - (int64_t)sc[j];
                const int dclip = delta < (int64_t)hp.c_int ? (int)delta : hp.c_int;
                idx = index_any(hp, -dclip, (uint32_t)p.top);
                sum += lut_b[idx];
            }
            w |= idx << (8 * j);
        }
        p.dec_idx[base * 2 * R * 4 + q] = (int32_t)w;
        atomicAdd(sums + n, sum); // LDS
    }
    __syncthreads();
    // one partial sum per workgroup; the other three slots of the chunk stay zero
    if (tid < 4 * R) p.dec_psum[((int64_t)grp * p.dec_np + chunk * 4 + tid / R) * R + tid % R] = tid < R ? (int32_t)sums[tid] : 0;
}

template <int D>
__global__ __launch_bounds__(NT) void decode_pv_kernel(const FwdParams p)
{
    constexpr int CB = D / 32;
    __shared__ __attribute__((aligned(1024))) int8_t Vs0[BK * D];
    __shared__ __attribute__((aligned(1024))) int8_t Vs1[BK * D];
    __shared__ int32_t row_sum[32];
    __shared__ uint32_t lut_lds[16];
    __shared__ uint8_t PT[31][68]; // per packed row: byte P - 128 of table index 0..64 (64 = hidden key, P = 0)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32, nt = nt32 / 4;
    const int t0 = chunk * p.dec_tpw, t1 = min(t0 + p.dec_tpw, nt);
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];
    stage_tile<D, true>(Vp, p.vs[2], p.Lk, t0, Vs0, wave, lane);
    if (tid < 16) lut_lds[tid] = p.lut[tid];
    reduce_partials<false>(p.dec_psum + (int64_t)grp * p.dec_np * R, p.dec_np, R, row_sum, tid); // ends with a barrier: lut_lds is visible

    if (p.dbg_row_sum && chunk == 0 && tid < R) {
        const RowOf ro = row_of(p, kvh, tid);
        p.dbg_row_sum[(int64_t)(b * p.Hq + ro.hq) * p.L + ro.i] = row_sum[tid];
    }
    // Eq. uint8-prob once per row and table entry: P = round(255 LUT_hat[idx] / S), exact
    for (int e = tid; e < R * 65; e += NT) {
        const int r = e / 65, idx = e % 65;
        const uint32_t S = (uint32_t)row_sum[r]; // >= 255: the key of the row maximum is visible
        const uint32_t ev = idx < 64 ? ((const uint8_t *)lut_lds)[idx] : 0u;
        PT[r][idx] = (uint8_t)((((510u * ev + S) / (2u * S)) ^ 0x80u) & 0xffu);
    }
    publish_tiles_barrier(); // the tables, and V tile t0 (requested at the top) are in LDS
    const uint8_t *pt = PT[n < R ? n : 0];
    // address of the transposing LDS read of V^T fragments within a 32-key sub-tile
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1, jj = tr_i >> 1;
    const int key = 8 * (jj >> 2) + 4 * h + (jj & 3);
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0;

    auto step = [&](int t, const int8_t *cur, int8_t *nxt) __attribute__((always_inline)) {
        if (t + 1 < t1) stage_tile<D, true>(Vp, p.vs[2], p.Lk, t + 1, nxt, wave, lane);
        // the lane's 16 probabilities as bytes P - 128; row 31 is all ones
        const int t32 = t * 4 + wave;
        v4i pf = {0, 0, 0, 0};
        if (n < R) {
            const v4i iw = *(const v4i *)(p.dec_idx + ((((int64_t)grp * nt32 + t32) * 2 + h) * R + n) * 4);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t wq = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) wq |= (uint32_t)pt[((uint32_t)iw[g] >> (8 * j)) & 0xffu] << (8 * j);
                pf[g] = (int)wq;
            }
        } else if (n == 31) {
            pf = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
        }
        const int8_t *Vsub = cur + wave * 32 * D;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int off = key * D + (((2 * cb + tr_g) ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
            const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off));
            const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off + 16 * D));
            const v4i vf = v4i{x0[0], x0[1], x1[0], x1[1]};
            o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, o[cb], 0, 0, 0);
        }
        publish_tiles_barrier(); // the next tile has arrived, and every wave is done with this one
    };
    for (int t = t0; t < t1; t += 2) {
        step(t, Vs0, Vs1);
        if (t + 1 < t1) step(t + 1, Vs1, Vs0);
    }

    // The four waves' sums meet in LDS (the V buffers are free now).  Register 4g + r of lane (n, h):
    // row n, channel 32 cb + 8 g + 4 h + r; row 31 holds the column sums of V over the wave's keys.
    int32_t *part = (int32_t *)Vs0; // 31 * D words fit: BK * D bytes = 32 * D words
    for (int e = tid; e < R * D; e += NT) part[e] = 0;
    __syncthreads();
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int32_t cs = __shfl(o[cb][i], 31 + 32 * h);
            if (n < R) atomicAdd(part + n * D + cb * 32 + 8 * (i >> 2) + 4 * h + (i & 3), o[cb][i] + 128 * cs); // LDS
        }
    __syncthreads();
    int32_t *dst = p.dec_acc + ((int64_t)grp * (p.dec_np / 4) + chunk) * R * D;
    for (int e = tid; e < R * D; e += NT) dst[e] = part[e];
}

// One workgroup per output row: sum of the tiles' partial accumulators (thread = four channels of
// every (NT / (D/4))-th tile, then an LDS reduction), requantization to INT8 (Sec. 3.2).
template <int D>
__global__ __launch_bounds__(NT) void decode_finish_kernel(const FwdParams p)
{
    constexpr int TPR = D / 4;    // threads per pass over the row's channels
    constexpr int TL = NT / TPR;  // tiles in flight
    __shared__ int32_t red[TL][D];
    const int row = blockIdx.x; // (b * Hq + hq) * L + i
    const int c0 = (threadIdx.x % TPR) * 4, tl = threadIdx.x / TPR;
    const int i = row % p.L, bh = row / p.L, hq = bh % p.Hq, b = bh / p.Hq;
    const int kvh = hq / p.group, r = (hq % p.group) * p.L + i, R = p.dec_rows, nt = p.dec_np / 4; // chunks
    const int32_t *src = p.dec_acc + (((int64_t)(b * p.Hkv + kvh) * nt) * R + r) * D + c0;
    v4i a = {0, 0, 0, 0};
#pragma unroll 8
    for (int t = tl; t < nt; t += TL) a += *(const v4i *)(src + (int64_t)t * R * D);
    *(v4i *)&red[tl][c0] = a;
    __syncthreads();
    if (tl != 0) return;
#pragma unroll
    for (int k = 1; k < TL; ++k) a += *(const v4i *)&red[k][c0];
    const HeadParams hp = p.hp_table[hq];
    const int64_t half = 1ll << (hp.rq_shift - 1);
    uint32_t packed = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (p.dbg_acc) p.dbg_acc[(int64_t)row * D + c0 + q] = a[q];
        int64_t v = ((int64_t)a[q] * hp.rq_mult + half) >> hp.rq_shift;
        v = v > 127 ? 127 : (v < -127 ? -127 : v);
        packed |= ((uint32_t)(int)v & 0xffu) << (8 * q);
    }
    *(uint32_t *)(p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)i * p.os[2] + c0) = packed;
}

template <int D>
int launch_d(const FwdParams &p, hipStream_t st)
{
    const dim3 grid((unsigned)(p.dec_np / 4), (unsigned)(p.B * p.Hkv)), block(NT);
    hipLaunchKernelGGL(decode_scores_kernel<D>, grid, block, 0, st, p);
    hipLaunchKernelGGL(decode_lookup_kernel, grid, block, 0, st, p);
    hipLaunchKernelGGL(decode_pv_kernel<D>, grid, block, 0, st, p);
    hipLaunchKernelGGL(decode_finish_kernel<D>, dim3((unsigned)(p.B * p.Hq * p.L)), block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// Packed rows (Hq / Hkv) * L must be at most 31, B * Hkv at most 65535; p.hp_table must hold every
// head's parameters with its index-map scheme in pad[0]; the dec_* workspace pointers must be set.
int launch_decode(const FwdParams &p, int d, void *stream)
{
    if (p.dec_rows < 1 || p.dec_rows > 31 || p.dec_tpw < 1 || !p.hp_table || (int64_t)p.B * p.Hkv > 65535) return (int)hipErrorInvalidValue;
    if (d == 64) return launch_d<64>(p, (hipStream_t)stream);
    if (d == 128) return launch_d<128>(p, (hipStream_t)stream);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
