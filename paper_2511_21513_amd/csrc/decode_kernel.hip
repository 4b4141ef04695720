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
// a workgroup walks tiles of 128 keys: one 32-key sub-tile per wave

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

// Workgroup barrier that orders LDS accesses only: global loads requested before it stay in flight across it
// (__syncthreads() waits for them).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// max (IS_MAX) or sum over all 32-key sub-tiles of the per-tile partials of every packed row, in two steps so
// that a kernel can put its own requests between the load and its use.  src is [nt32][R].  Thread tid takes row
// tid % R of every (NT / R)-th sub-tile (several loads in flight each) ...
template <bool IS_MAX>
__device__ __forceinline__ int32_t partial_of_thread(const int32_t *src, int nt32, int R, int tid)
{
    const int per = NT / R; // sub-tiles covered per pass
    int32_t v = IS_MAX ? INT32_MIN : 0;
    if (tid < per * R) {
        const int r = tid % R;
        if (nt32 <= per) { // one load per thread, and no loop (in front of a loop the compiler waits for every load in flight)
            if (tid / R < nt32) v = src[(int64_t)(tid / R) * R + r];
        } else {
#pragma unroll 8
            for (int j = tid / R; j < nt32; j += per) {
                const int32_t x = src[(int64_t)j * R + r];
                v = IS_MAX ? max(v, x) : v + x;
            }
        }
    }
    return v;
}
// ... then one LDS atomic per thread: red[r] for r < R.  Ends with a barrier.
template <bool IS_MAX>
__device__ __forceinline__ void reduce_partials(int32_t v, int R, int32_t *red, int tid)
{
    if (tid < 32) red[tid] = IS_MAX ? INT32_MIN : 0;
    lds_barrier();
    if (tid < (NT / R) * R) {
        if (IS_MAX) atomicMax(red + tid % R, v);
        else atomicAdd(red + tid % R, v);
    }
    lds_barrier();
}

// The three kernels below share a grid: x = chunk of p.dec_tpw consecutive 128-key tiles,
// y = b * Hkv + kvh.  Partial row maxima and sums are kept per (chunk, wave): np = 4 * chunks per row.

// Streams K straight from global memory into the MFMA operand registers: lane (n, h) of a wave reads, for
// every 32-channel block, the 16 bytes of key row n that its operand holds.  No LDS and no workgroup barrier;
// wave w of the workgroup takes sub-tile w of every 128-key tile of the chunk, with the rows of the next
// KDEPTH - 1 sub-tiles in flight (register sets named statically, so that a wait covers one set only).
template <int D>
__global__ __launch_bounds__(NT) void decode_scores_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32, nt = nt32 / 4;
    const int t0 = chunk * p.dec_tpw, t1 = min(t0 + p.dec_tpw, nt);
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    // Key rows at or past Lk: the last row is read instead; their scores are hidden keys and never used.  Past the
    // end of the chunk the last sub-tile is requested again (and never used): no branch around the loads.
    auto load_kf = [&](int t, v4i (&kf)[KB]) __attribute__((always_inline)) {
        const int key = min((min(t, t1 - 1) * 4 + wave) * 32 + n, p.Lk - 1);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = *(const v4i *)(Kp + (int64_t)key * p.ks[2] + kb * 32 + h * 16);
    };
    // Q fragments: packed row n, bytes [32 kb + 16 h, +16); lanes of unused operand rows hold row R - 1 again
    // (their scores are never stored).  Requested before K, so that the first wait for K covers them.
    const RowOf ro = row_of(p, kvh, min(n, R - 1));
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
        qf[kb] = *(const v4i *)(p.q + (int64_t)b * p.qs[0] + (int64_t)ro.hq * p.qs[1] + (int64_t)ro.i * p.qs[2] + kb * 32 + h * 16);
    v4i kA[KB], kB[KB], kC[KB];
    load_kf(t0, kA);
    load_kf(t0 + 1, kB);
    load_kf(t0 + 2, kC);
    int32_t m = INT32_MIN;
    __shared__ __attribute__((aligned(16))) int32_t stage_all[WAVES][32 * 32];
    int32_t *stage = &stage_all[wave][0];
    auto body = [&](int t, const v4i (&kf)[KB]) __attribute__((always_inline)) {
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[kb], s, 0, 0, 0);
        // register i of lane (n, h): packed row n, key key0 + acc_key(i, h)
        const int t32 = t * 4 + wave, key0 = t32 * 32;
        if (key0 + 32 <= p.Lk && (!p.causal || key0 + 31 <= p.row_lo)) { // every key visible to every row
#pragma unroll
            for (int i = 0; i < 16; i += 2) m = max(max(s[i], s[i + 1]), m);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (key_visible(p, key0 + acc_key(i, h), ro.i)) m = max(m, s[i]);
        }
        // The scores of the sub-tile, [h][row][16], are contiguous in memory (128 R bytes) but sit in 2 R lanes.
        // They pass through a wave-private LDS buffer so that every store instruction writes whole lines, 16
        // bytes per lane (stores of 16 bytes at a stride of 64 cost a third of the kernel's time).  The LDS
        // executes a wave's instructions in order: no barrier.
        if (n < R) {
#pragma unroll
            for (int g = 0; g < 4; ++g) *(v4i *)(stage + (h * R + n) * 16 + 4 * g) = v4i{s[4 * g], s[4 * g + 1], s[4 * g + 2], s[4 * g + 3]};
        }
        int32_t *dst = p.dec_scores + ((int64_t)grp * nt32 + t32) * 2 * R * 16;
        for (int q = lane; q < 8 * R; q += 64) *(v4i *)(dst + 4 * q) = *(const v4i *)(stage + 4 * q);
    };
    // no branch inside the loop: a path that skips a request would make every wait of the loop conservative
    int t = t0;
    for (; t + 2 < t1; t += 3) {
        body(t, kA);
        load_kf(t + 3, kA);
        body(t + 1, kB);
        load_kf(t + 4, kB);
        body(t + 2, kC);
        load_kf(t + 5, kC);
    }
    if (t < t1) body(t, kA);
    if (t + 1 < t1) body(t + 1, kB);
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
    reduce_partials<true>(partial_of_thread<true>(p.dec_pmax + (int64_t)grp * p.dec_np * R, p.dec_np, R, tid), R, row_max, tid);
    if (p.dbg_row_max && chunk == 0 && tid < R) {
        const RowOf ro = row_of(p, kvh, tid);
        p.dbg_row_max[(int64_t)(b * p.Hq + ro.hq) * p.L + ro.i] = row_max[tid];
    }
    const uint8_t *lut_b = (const uint8_t *)lut_lds;
    // group q of four scores: q = ((sub-tile * 2 + h) * R + n) * 4 + g holds registers 4g .. 4g+3 of lane (n, h)
    const int64_t base = (int64_t)grp * nt32 + (int64_t)t0 * 4; // first sub-tile of the chunk
    const int nq = (t1 - t0) * 4 * 2 * R * 4;
    constexpr int UN = 8; // loads in flight per thread
    for (int q0 = 0; q0 < nq; q0 += UN * NT) {
        v4i scs[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int q = q0 + u * NT + tid;
            scs[u] = v4i{0, 0, 0, 0};
            if (q < nq) scs[u] = *(const v4i *)(p.dec_scores + (base * 2 * R * 4 + q) * 4);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int q = q0 + u * NT + tid;
            if (q >= nq) break;
            const v4i sc = scs[u];
            const int g = q & 3, rn = q >> 2, n = rn % R, sh = rn / R, h = sh & 1, t32l = sh >> 1;
            const int key0 = (t0 * 4 + t32l) * 32;
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
    }
    __syncthreads();
    // one partial sum per workgroup; the other three slots of the chunk stay zero
    if (tid < 4 * R) p.dec_psum[((int64_t)grp * p.dec_np + chunk * 4 + tid / R) * R + tid % R] = tid < R ? (int32_t)sums[tid] : 0;
}

// Streams V through registers: a wave reads its 32-key sub-tile row by row (whole rows, coalesced), with the
// next sub-tile and its table indices in flight, writes it to a wave-private LDS buffer (chunks of 16 bytes
// XOR-swizzled) and takes the V^T operand from there with the transposing read.  The LDS executes one wave's
// instructions in order, so no barrier separates a wave's writes from its reads.
template <int D>
__global__ __launch_bounds__(NT, 4) void decode_pv_kernel(const FwdParams p)
{
    constexpr int CB = D / 32;
    constexpr int NBLK = 32 * D / 1024, CPR = D / 16, RPB = 1024 / D; // 1 KiB blocks of a sub-tile: one wave-wide 16-byte load each
    __shared__ __attribute__((aligned(1024))) int8_t Vw[WAVES][32 * D];
    __shared__ int32_t row_sum[32];
    __shared__ uint32_t lut_lds[16];
    __shared__ uint8_t PT[31][68]; // per packed row: byte P - 128 of table index 0..64 (64 = hidden key, P = 0)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv;
    const int R = p.dec_rows, nt32 = p.dec_nt32, nt = nt32 / 4;
    const int t0 = chunk * p.dec_tpw, t1 = min(t0 + p.dec_tpw, nt);
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];
    struct Sub {
        v4i v[NBLK]; // block j: key row j * RPB + lane / CPR of the sub-tile, chunk lane % CPR
        v4i iw;      // table indices of lane (n, h), 16 bytes
    };
    // Key rows at or past Lk: the last row is read instead.  Such keys are hidden (byte -128), and the
    // correction 128 * colsum is taken from the same operand, so whatever V holds there cancels exactly.
    // Past the end of the chunk the last sub-tile is requested again (and never used), so that the loop body
    // holds no branch around its loads; lanes of unused operand rows read the indices of row R - 1.
    auto load_sub = [&](int t, Sub &x) __attribute__((always_inline)) {
        const int t32 = min(t, t1 - 1) * 4 + wave;
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            const int key = min(t32 * 32 + j * RPB + lane / CPR, p.Lk - 1);
            x.v[j] = *(const v4i *)(Vp + (int64_t)key * p.vs[2] + (lane % CPR) * 16);
        }
        x.iw = *(const v4i *)(p.dec_idx + ((((int64_t)grp * nt32 + t32) * 2 + h) * R + min(n, R - 1)) * 4);
    };
    Sub sA, sB;
    // the small loads first: loads return in the order of their requests
    if (tid < 16) lut_lds[tid] = p.lut[tid];
    const int32_t my_sum = partial_of_thread<false>(p.dec_psum + (int64_t)grp * p.dec_np * R, p.dec_np, R, tid);
    load_sub(t0, sA);
    load_sub(t0 + 1, sB);
    reduce_partials<false>(my_sum, R, row_sum, tid); // ends with a barrier: lut_lds is visible

    if (p.dbg_row_sum && chunk == 0 && tid < R) {
        const RowOf ro = row_of(p, kvh, tid);
        p.dbg_row_sum[(int64_t)(b * p.Hq + ro.hq) * p.L + ro.i] = row_sum[tid];
    }
    // Eq. uint8-prob once per row and table entry: P = round(255 LUT_hat[idx] / S), exact
    for (int e = tid; e < R * 65; e += NT) {
        const int r = e / 65, idx = e % 65;
        const uint32_t S = (uint32_t)row_sum[r]; // >= 255: the key of the row maximum is visible
        const uint32_t ev = idx < 64 ? ((const uint8_t *)lut_lds)[idx] : 0u;
        PT[r][idx] = (uint8_t)((prob_u8(ev, S, __builtin_amdgcn_rcpf((float)(2u * S))) ^ 0x80u) & 0xffu);
    }
    lds_barrier(); // the tables are in LDS
    const uint8_t *pt = PT[n < R ? n : 0];
    int8_t *Vsub = &Vw[wave][0];
    // where this lane's rows go: block j holds key row j * RPB + lane / CPR
    const int wkey = lane / CPR, wcp = lane % CPR;
    // address of the transposing LDS read of V^T fragments within a 32-key sub-tile
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1, jj = tr_i >> 1;
    const int key = 8 * (jj >> 2) + 4 * h + (jj & 3);
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0;

    auto body = [&](const Sub &x) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            const int kr = j * RPB + wkey;
            *(v4i *)(Vsub + kr * D + ((wcp ^ swz_v<D>(kr)) << 4)) = x.v[j];
        }
        // the lane's 16 probabilities as bytes P - 128; row 31 is all ones
        v4i pf = {0, 0, 0, 0};
        if (n < R) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t wq = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) wq |= (uint32_t)pt[((uint32_t)x.iw[g] >> (8 * j)) & 0xffu] << (8 * j);
                pf[g] = (int)wq;
            }
        } else if (n == 31) {
            pf = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int off = key * D + (((2 * cb + tr_g) ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
            const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off));
            const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off + 16 * D));
            const v4i vf = v4i{x0[0], x0[1], x1[0], x1[1]};
            o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, o[cb], 0, 0, 0);
        }
    };
    // no branch inside the loop: a path that skips a request would make every wait of the loop conservative
    int t = t0;
    for (; t + 1 < t1; t += 2) {
        body(sA);
        load_sub(t + 2, sA);
        body(sB);
        load_sub(t + 3, sB);
    }
    if (t < t1) body(sA);
    __syncthreads(); // every wave is done with its V buffer

    // The four waves' sums meet in LDS (the V buffers are free now).  Register 4g + r of lane (n, h):
    // row n, channel 32 cb + 8 g + 4 h + r; row 31 holds the column sums of V over the wave's keys.
    int32_t *part = (int32_t *)&Vw[0][0]; // R + 1 <= 32 rows of D words fit: the four buffers hold 128 * D bytes
    for (int e = tid; e < (R + 1) * D; e += NT) part[e] = 0;
    __syncthreads();
    if (n < R || n == 31) { // row R of `part` takes the column sums
        int32_t *dstl = part + (n < R ? n : R) * D + 4 * h;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) atomicAdd(dstl + cb * 32 + 8 * (i >> 2) + (i & 3), o[cb][i]); // LDS
    }
    __syncthreads();
    int32_t *dst = p.dec_acc + ((int64_t)grp * (p.dec_np / 4) + chunk) * R * D;
    for (int e = tid; e < R * D; e += NT) dst[e] = part[e] + 128 * part[R * D + e % D];
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
    uint32_t packed = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (p.dbg_acc) p.dbg_acc[(int64_t)row * D + c0 + q] = a[q];
        packed |= ((uint32_t)requant_any(a[q], hp.rq_mult, hp.rq_shift) & 0xffu) << (8 * q);
    }
    *(uint32_t *)(p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)i * p.os[2] + c0) = packed;
}

// ---------------------------------------------------------------------------------------------------------
// The same three reductions in ONE launch.  The workgroups of a (batch, KV head) group (consecutive ids: they are
// dispatched together) meet twice at a counter of their own in device memory -- after the row maxima, after the
// row sums -- so the scores and table indices of a chunk never leave the workgroup's LDS and HBM sees K, V, Q,
// the output and the partial accumulators only.  A score is kept as a 16-bit distance below the row maximum of
// its own 32-key sub-tile (saturated at 65535; the sub-tile's maximum is kept beside it): with the global row
// maximum M, Delta = (M - sub-tile maximum) + distance, and a saturated distance is past every clip threshold
// up to 65535, which the host checks.  WIDE: the raw 32-bit scores instead, for thresholds that are larger or
// known on the device only; the chunk a workgroup can hold is then half as long.  Waiting is bounded: a workgroup whose group does not arrive within
// dec_spin_limit polls raises the group's status word and returns, so the grid always drains.
// The last workgroup of a group to finish adds up the partial accumulators, requantizes, and clears the group's state.
__device__ __forceinline__ uint32_t bias_i32(int32_t x) { return (uint32_t)x ^ 0x80000000u; }
__device__ __forceinline__ int32_t unbias_i32(uint32_t u) { return (int32_t)(u ^ 0x80000000u); }

// Arrival at the group's counter, then wait until `target` arrivals; false after `limit` polls.  Everything the
// workgroups of a group exchange goes through device-scope atomics (performed at the coherence point, past the
// per-XCD L2), so no cache write-back or invalidation is needed: a thread only waits until its own atomics have
// been performed before the workgroup arrives.  (Fences at device scope write back and invalidate the whole L2
// of the XCD; with a thousand workgroups meeting twice they took 1 ms.)
__device__ __forceinline__ bool group_meet(uint32_t *ctr, uint32_t target, int limit, int tid, int32_t *flag)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    if (tid == 0) {
        atomicAdd(ctr, 1u);
        int it = 0, ok = 1;
        while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(4);
            if (++it > limit) {
                ok = 0;
                break;
            }
        }
        *flag = ok;
    }
    lds_barrier();
    return *flag != 0;
}

template <int D, bool WIDE>
__global__ __launch_bounds__(NT, 4) void decode_fused_kernel(const FwdParams p)
{
    constexpr int KB = D / 32, CB = D / 32;
    constexpr int NBLK = 32 * D / 1024, CPR = D / 16, RPB = 1024 / D;
    constexpr int UW = WIDE ? 4 : 2; // words per unit of four scores
    // 16 KiB: 4 tpw * 2 R * 4 units, i.e. R * tpw <= 64 (32 when WIDE); [sub-tile][h][row][16] distances of 16 bits
    // each (scores of 32 when WIDE); later the first word of every unit holds its four table indices
    __shared__ __attribute__((aligned(16))) uint32_t sc16[4096];
    __shared__ __attribute__((aligned(1024))) int8_t Vw[WAVES][32 * D];
    __shared__ int32_t sub_max[256]; // [sub-tile][row]: 4 tpw * R <= 256 entries
    __shared__ int32_t row_max[32], row_sum[32], row_i[32], meet_flag;
    __shared__ HeadParams row_hp[32];
    __shared__ uint32_t lut_lds[16];
    __shared__ uint8_t PT[31][68];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x, grp = blockIdx.y, b = grp / p.Hkv, kvh = grp % p.Hkv, C = gridDim.x;
    const int R = p.dec_rows, nt32 = p.dec_nt32, nt = nt32 / 4;
    const int t0 = chunk * p.dec_tpw, t1 = min(t0 + p.dec_tpw, nt);
    uint32_t *state = p.dec_state + (int64_t)grp * DEC_STATE_WORDS;
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    // ================================================================ scores (Sec. 2.1), row maxima (Sec. 3.1)
    const RowOf ro = row_of(p, kvh, min(n, R - 1));
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
        qf[kb] = *(const v4i *)(p.q + (int64_t)b * p.qs[0] + (int64_t)ro.hq * p.qs[1] + (int64_t)ro.i * p.qs[2] + kb * 32 + h * 16);
    auto load_kf = [&](int t, v4i (&kf)[KB]) __attribute__((always_inline)) {
        const int key = min((min(t, t1 - 1) * 4 + wave) * 32 + n, p.Lk - 1);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = *(const v4i *)(Kp + (int64_t)key * p.ks[2] + kb * 32 + h * 16);
    };
    v4i kA[KB], kB[KB], kC[KB];
    load_kf(t0, kA);
    load_kf(t0 + 1, kB);
    load_kf(t0 + 2, kC);
    if (tid < 16) lut_lds[tid] = p.lut[tid];
    if (tid < 32) {
        row_max[tid] = INT32_MIN;
        row_sum[tid] = 0;
        if (tid < R) {
            const RowOf r2 = row_of(p, kvh, tid);
            row_i[tid] = r2.i;
            row_hp[tid] = p.hp_table[r2.hq];
        }
    }
    int32_t m = INT32_MIN;
    auto score_body = [&](int t, const v4i (&kf)[KB]) __attribute__((always_inline)) {
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[kb], s, 0, 0, 0);
        const int tl = (t - t0) * 4 + wave, key0 = (t * 4 + wave) * 32; // sub-tile within the chunk, its first key
        const bool full = key0 + 32 <= p.Lk && (!p.causal || key0 + 31 <= p.row_lo); // every key visible to every row
        int32_t sm = INT32_MIN;
        if (full) {
#pragma unroll
            for (int i = 0; i < 16; i += 2) sm = max(max(s[i], s[i + 1]), sm);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (key_visible(p, key0 + acc_key(i, h), ro.i)) sm = max(sm, s[i]);
        }
        sm = max(sm, __shfl_xor(sm, 32));
        m = max(m, sm);
        if (WIDE) {
            if (n < R) {
                uint32_t *dst = sc16 + ((tl * 2 + h) * R + n) * 16;
#pragma unroll
                for (int g = 0; g < 4; ++g) *(v4i *)(dst + 4 * g) = v4i{s[4 * g], s[4 * g + 1], s[4 * g + 2], s[4 * g + 3]};
            }
            return;
        }
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            // hidden keys get the saturated distance too (the lookup decides on visibility by the key number)
            uint32_t d0 = 65535u, d1 = 65535u;
            if (full || key_visible(p, key0 + acc_key(i, h), ro.i)) d0 = min((uint32_t)(sm - s[i]), 65535u);
            if (full || key_visible(p, key0 + acc_key(i + 1, h), ro.i)) d1 = min((uint32_t)(sm - s[i + 1]), 65535u);
            w[i / 2] = d0 | (d1 << 16);
        }
        if (n < R) {
            uint32_t *dst = sc16 + ((tl * 2 + h) * R + n) * 8;
            *(v4i *)dst = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            *(v4i *)(dst + 4) = v4i{(int)w[4], (int)w[5], (int)w[6], (int)w[7]};
            if (h == 0) sub_max[tl * R + n] = sm;
        }
    };
    {
        int t = t0;
        for (; t + 2 < t1; t += 3) {
            score_body(t, kA);
            load_kf(t + 3, kA);
            score_body(t + 1, kB);
            load_kf(t + 4, kB);
            score_body(t + 2, kC);
            load_kf(t + 5, kC);
        }
        if (t < t1) score_body(t, kA);
        if (t + 1 < t1) score_body(t + 1, kB);
    }
    lds_barrier(); // row_max[] is initialised
    if (n < R && h == 0) atomicMax(row_max + n, m); // LDS
    lds_barrier();
    if (tid < R) atomicMax(state + 32 + tid, bias_i32(row_max[tid]));

    // V of the first two sub-tiles is requested before the meetings: it travels while the group gathers
    struct Sub {
        v4i v[NBLK]; // block j: key row j * RPB + lane / CPR of the sub-tile, chunk lane % CPR
    };
    auto load_sub = [&](int t, Sub &x) __attribute__((always_inline)) {
        const int t32 = min(t, t1 - 1) * 4 + wave;
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            const int key = min(t32 * 32 + j * RPB + lane / CPR, p.Lk - 1);
            x.v[j] = *(const v4i *)(Vp + (int64_t)key * p.vs[2] + (lane % CPR) * 16);
        }
    };
    if (!group_meet(state + 0, (uint32_t)C, p.dec_spin_limit, tid, &meet_flag)) {
        if (tid == 0) atomicOr(state + 2, 1u);
        return;
    }
    Sub sA, sB;
    load_sub(t0, sA);
    load_sub(t0 + 1, sB);
    if (tid < R) {
        row_max[tid] = unbias_i32(__hip_atomic_load(state + 32 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if (p.dbg_row_max && chunk == 0) p.dbg_row_max[(int64_t)(b * p.Hq + kvh * p.group + tid / p.L) * p.L + tid % p.L] = row_max[tid];
    }
    lds_barrier();

    // ================================================================ table indices (Eq. int_clipping, Eq. gather16), row sums
    {
        const uint8_t *lut_b = (const uint8_t *)lut_lds;
        const int nq = (t1 - t0) * 4 * 2 * R * 4; // units of four scores: q = ((sub-tile * 2 + h) * R + row) * 4 + g
        int acc_row = -1; // a thread's sums go to LDS when its row changes (never, where R divides 64)
        uint32_t acc = 0;
        for (int q = tid; q < nq; q += NT) {
            const int g = q & 3, rn = q >> 2, nn = rn % R, sh = rn / R, hh = sh & 1, tl = sh >> 1;
            const int key0 = (t0 * 4 + tl) * 32;
            uint32_t u[4]; // the unit's distances (WIDE: its raw scores)
            if (WIDE) {
                const v4i x = *(const v4i *)(sc16 + 4 * q);
                u[0] = (uint32_t)x[0], u[1] = (uint32_t)x[1], u[2] = (uint32_t)x[2], u[3] = (uint32_t)x[3];
            } else {
                const uint32_t lo = sc16[2 * q], hi = sc16[2 * q + 1];
                u[0] = lo & 0xffffu, u[1] = lo >> 16, u[2] = hi & 0xffffu, u[3] = hi >> 16;
            }
            // >= 0 and below 2^23 where the row sees a key of the sub-tile (meaningless, and unused, where it sees none)
            const int base = WIDE ? row_max[nn] : (int)((uint32_t)row_max[nn] - (uint32_t)sub_max[tl * R + nn]);
            const int ri = row_i[nn];
            const HeadParams &hp = row_hp[nn];
            const bool full = key0 + 32 <= p.Lk && (!p.causal || key0 + 31 <= p.row_lo + ri);
            uint32_t w = 0, sum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t idx = 64u; // hidden key: probability 0
                if (full || key_visible(p, key0 + acc_key(4 * g + j, hh), ri)) {
                    const int delta = WIDE ? base - (int)u[j] : base + (int)u[j]; // scores are below 2^22 in magnitude
                    idx = index_any(hp, -min(delta, hp.c_int), (uint32_t)p.top);
                    sum += lut_b[idx];
                }
                w |= idx << (8 * j);
            }
            sc16[UW * q] = w; // the unit's first word now holds its four indices
            if (nn != acc_row) {
                if (acc_row >= 0) atomicAdd(row_sum + acc_row, (int32_t)acc); // LDS
                acc_row = nn;
                acc = 0;
            }
            acc += sum;
        }
        if (acc_row >= 0) atomicAdd(row_sum + acc_row, (int32_t)acc); // LDS
    }
    lds_barrier();
    if (tid < R) atomicAdd(state + 64 + tid, (uint32_t)row_sum[tid]);
    if (!group_meet(state + 0, (uint32_t)(2 * C), p.dec_spin_limit, tid, &meet_flag)) {
        if (tid == 0) atomicOr(state + 2, 1u);
        return;
    }
    if (tid < R) {
        row_sum[tid] = (int32_t)__hip_atomic_load(state + 64 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p.dbg_row_sum && chunk == 0) p.dbg_row_sum[(int64_t)(b * p.Hq + kvh * p.group + tid / p.L) * p.L + tid % p.L] = row_sum[tid];
    }
    lds_barrier();
    // Eq. uint8-prob once per row and table entry: P = round(255 LUT_hat[idx] / S), exact
    for (int e = tid; e < R * 65; e += NT) {
        const int r = e / 65, idx = e % 65;
        const uint32_t S = (uint32_t)row_sum[r]; // >= 255: the key of the row maximum is visible
        const uint32_t ev = idx < 64 ? ((const uint8_t *)lut_lds)[idx] : 0u;
        PT[r][idx] = (uint8_t)((prob_u8(ev, S, __builtin_amdgcn_rcpf((float)(2u * S))) ^ 0x80u) & 0xffu);
    }
    lds_barrier();

    // ================================================================ P_hat V_hat (Sec. 3.2)
    const uint8_t *pt = PT[n < R ? n : 0];
    int8_t *Vsub = &Vw[wave][0];
    const int wkey = lane / CPR, wcp = lane % CPR;
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1, jj = tr_i >> 1;
    const int key = 8 * (jj >> 2) + 4 * h + (jj & 3);
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0;
    auto pv_body = [&](int t, const Sub &x) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            const int kr = j * RPB + wkey;
            *(v4i *)(Vsub + kr * D + ((wcp ^ swz_v<D>(kr)) << 4)) = x.v[j];
        }
        v4i pf = {0, 0, 0, 0};
        if (n < R) {
            const uint32_t *iw = sc16 + ((((t - t0) * 4 + wave) * 2 + h) * R + n) * 4 * UW; // index words of the lane's four units
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t ix = iw[UW * g];
                uint32_t wq = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) wq |= (uint32_t)pt[(ix >> (8 * j)) & 0xffu] << (8 * j);
                pf[g] = (int)wq;
            }
        } else if (n == 31) {
            pf = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int off = key * D + (((2 * cb + tr_g) ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
            const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off));
            const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + off + 16 * D));
            const v4i vf = v4i{x0[0], x0[1], x1[0], x1[1]};
            o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, o[cb], 0, 0, 0);
        }
    };
    {
        int t = t0;
        for (; t + 1 < t1; t += 2) {
            pv_body(t, sA);
            load_sub(t + 2, sA);
            pv_body(t + 1, sB);
            load_sub(t + 3, sB);
        }
        if (t < t1) pv_body(t, sA);
    }
    lds_barrier(); // every wave is done with its V buffer

    // the four waves' sums meet in LDS; row 31 of the operand holds the column sums of V over the wave's keys
    int32_t *part = (int32_t *)&Vw[0][0]; // R + 1 <= 32 rows of D words fit: the four buffers hold 128 * D bytes
    for (int e = tid; e < (R + 1) * D; e += NT) part[e] = 0;
    lds_barrier();
    if (n < R || n == 31) { // row R of `part` takes the column sums
        int32_t *dst = part + (n < R ? n : R) * D + 4 * h;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) atomicAdd(dst + cb * 32 + 8 * (i >> 2) + (i & 3), o[cb][i]); // LDS
    }
    lds_barrier();
    int32_t *acc_grp = p.dec_acc + (int64_t)grp * C * R * D;
    // (device-scope stores and loads for what another workgroup reads: they pass the L2 of the XCD)
    for (int e = tid; e < R * D; e += NT)
        __hip_atomic_store(acc_grp + (int64_t)chunk * R * D + e, part[e] + 128 * part[R * D + e % D], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // departure: the last workgroup of the group finishes the rows
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    if (tid == 0) meet_flag = (int32_t)atomicAdd(state + 1, 1u);
    lds_barrier();
    if (meet_flag != C - 1) return;
    for (int e = tid; e < R * (D / 4); e += NT) {
        const int r = e / (D / 4), c0 = (e % (D / 4)) * 4;
        v4i a = {0, 0, 0, 0};
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                a[q] += __hip_atomic_load(acc_grp + ((int64_t)c * R + r) * D + c0 + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int hq = kvh * p.group + r / p.L, i = r % p.L;
        const HeadParams &hp = row_hp[r];
        uint32_t packed = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (p.dbg_acc) p.dbg_acc[((int64_t)(b * p.Hq + hq) * p.L + i) * D + c0 + q] = a[q];
            packed |= ((uint32_t)requant_any(a[q], hp.rq_mult, hp.rq_shift) & 0xffu) << (8 * q);
        }
        *(uint32_t *)(p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)i * p.os[2] + c0) = packed;
    }
    // the group's state back to zero for the next launch (status stays)
    if (tid < DEC_STATE_WORDS && tid != 2) __hip_atomic_store(state + tid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
int launch_d(const FwdParams &p, hipStream_t st)
{
    const dim3 grid((unsigned)(p.dec_np / 4), (unsigned)(p.B * p.Hkv)), block(NT);
    if (p.dec_state) {
        if (p.dec_rows * p.dec_tpw > (p.dec_wide ? 32 : 64)) return (int)hipErrorInvalidValue;
        if (p.dec_wide) hipLaunchKernelGGL((decode_fused_kernel<D, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((decode_fused_kernel<D, false>), grid, block, 0, st, p);
        return (int)hipGetLastError();
    }
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
