// Sweep C of the IntAttention forward as a kernel of its own (gfx950): with the row maxima and row
// sums of E_hat already in a workspace, recompute the INT8 scores, map them through the index
// map and the per-row probability table (Sec. 3.1-3.2: P_hat = round(255 E_hat / S)), multiply
// by V_hat on the matrix cores and requantize (INT8 output).
//
// Same data layout and lane ownership as the generic forward kernel (transposed scores, one query
// row per lane, 32 rows per wave, 4 waves per workgroup, XOR-swizzled K/V tiles in LDS filled by
// direct global->LDS loads).  What differs is the instruction schedule.  The generic kernel runs a
// tile as phases (scores, lookups, pack, P.V), so the matrix core idles during the vector phases
// and the other way round; two waves per SIMD do not hide that.  Here the key axis is walked in
// steps of 32 keys as a software pipeline inside each wave.  Step j issues, in this order,
//     one MFMA, then the vector work of two scores, one MFMA, ...:
//   MFMAs:   the KB chained MFMAs of the scores of sub-tile j+1, then the CB MFMAs P.V of sub-tile j-1
//   vector:  clip/index/table lookup (issued, not awaited) of sub-tile j's scores, and the packing
//            of sub-tile j-1's looked-up probability bytes into the MFMA operand (before its P.V)
//   LDS:     K fragments of sub-tile j+2 (once the current ones are consumed), V^T fragments of
//            sub-tile j (after the last P.V of j-1 has issued)
// so every MFMA runs under independent vector instructions of the same wave, every LDS result
// has a whole step to arrive, and nothing waits on what it has just issued.  Scheduling barriers
// pin that order.
//
// Tiles are 64 keys (two steps), double buffered per operand.  K is needed one tile before V
// (scores of tile T+1 are computed while tile T's probabilities meet V), so at the top of
// iteration T the loads of K tile T+2 and V tile T+1 are issued; one barrier per iteration.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;

template <int D, bool CAUSAL, int MODE>
__global__ __launch_bounds__(NT, 1) void sweep_c_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;       // 32-wide blocks of the head dimension
    constexpr int CB = D / 32;       // 32-wide blocks of output channels
    constexpr int BK = 64;           // keys per tile: two pipeline steps
    constexpr int BQ = WAVES * 32;
    constexpr int TILE = BK * D;     // bytes
    constexpr int SUB = 32 * D;      // bytes of a 32-key sub-tile
    constexpr int NBLK = TILE / 1024;
    constexpr int JB = (NBLK + WAVES - 1) / WAVES;
    constexpr int CPR = D / 16;
    constexpr int RPB = 1024 / D;
    constexpr int NSLOT = KB + CB;   // MFMAs per step
    constexpr int EPS = 16 / NSLOT;  // scores handled after each MFMA
    constexpr int GPS = 4 / KB;      // operand registers packed after each of the first KB MFMAs
    static_assert(16 % NSLOT == 0 && 4 % KB == 0, "vector work must split evenly over the MFMA slots");

    __shared__ __attribute__((aligned(1024))) int8_t Ks0[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Ks1[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Vs0[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Vs1[TILE];
    __shared__ uint32_t PT[WAVES][32 * 32]; // [idx][row] per wave
    __shared__ uint32_t lut_lds[8];
    __shared__ int32_t colsum[D];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return; // padding of the XCD-aware grid (uniform for the whole workgroup)
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt;
    const int bh = b * p.Hq + hq;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    const int L = p.L;
    const uint32_t top = (uint32_t)p.top;

    const int q0 = qt * BQ, qw0 = q0 + wave * 32;
    const int row = qw0 + n; // this lane's query row
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    if (tid < 8) lut_lds[tid] = p.lut[tid];

    // Q fragments: row qw0 + n, bytes [32 kb + 16 h, +16)
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (row < L) qf[kb] = *(const v4i *)(Qp + (int64_t)row * p.qs[2] + kb * 32 + h * 16);
    }

    const int kmax = CAUSAL ? min(L, q0 + BQ) : L;
    const int ntiles = (kmax + BK - 1) / BK;

    // ---- staging: direct global -> LDS loads; the XOR swizzle is applied to the global address
    // (lane i of a wave-wide 16-byte load lands at byte 16 i of its 1 KiB block).
    int dma_goff_k[JB], dma_goff_v[JB];
#pragma unroll
    for (int j = 0; j < JB; ++j) {
        const int key = (wave + WAVES * j) * RPB + lane / CPR, cp = lane % CPR;
        dma_goff_k[j] = key * (int)p.ks[2] + ((cp ^ swz_k<D>(key)) << 4); // the host checked BK * stride < 2^31
        dma_goff_v[j] = key * (int)p.vs[2] + ((cp ^ swz_v<D>(key)) << 4);
    }
    // The loads go through a buffer descriptor that starts at the tile and ends with the last
    // byte of key row L-1, so key rows at or past L come back as zeros from the range check.
    auto dma_tile = [&](const int8_t *base, int64_t stride, const int (&goff)[JB], int t, int8_t *dst)
                        __attribute__((always_inline)) {
        const int8_t *tb = base + (int64_t)t * BK * stride; // wave-uniform
        const int64_t rem = (int64_t)(L - t * BK - 1) * stride + D;
        const uint32_t nrec = rem > 0xffffffffll ? 0xffffffffu : (uint32_t)rem;
#if defined(__HIP_DEVICE_COMPILE__) // the host pass has neither the descriptor type nor the builtins
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)tb, 0, (int)nrec, 0x00020000);
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int blk = wave + WAVES * j;
            if (NBLK % WAVES != 0 && blk >= NBLK) break;    // wave-uniform
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(dst + blk * 1024), 16,
                                                     goff[j], 0, 0, 0);
        }
#else
        (void)tb, (void)nrec, (void)goff, (void)dst;
#endif
    };
    auto dma_k = [&](int t, int8_t *dst) __attribute__((always_inline)) { dma_tile(Kp, p.ks[2], dma_goff_k, t, dst); };
    auto dma_v = [&](int t, int8_t *dst) __attribute__((always_inline)) { dma_tile(Vp, p.vs[2], dma_goff_v, t, dst); };

    dma_k(0, Ks0);
    dma_v(0, Vs0);
    if (ntiles > 1) dma_k(1, Ks1);

    // ---- per-row state from the first launch, probability table, column sums of V
    const int mx = row < L ? p.ws_row_max[(int64_t)bh * L + row] : 0;
    uint32_t sum = row < L ? (uint32_t)p.ws_row_sum[(int64_t)bh * L + row] : 0u;
    if (sum == 0) sum = 1; // only rows beyond L; never stored
    RowIndex<MODE> ri;
    ri.init(hp, mx, top);
    if (p.dbg_row_max && h == 0 && row < L) p.dbg_row_max[(int64_t)bh * L + row] = mx;
    if (p.dbg_row_sum && h == 0 && row < L) p.dbg_row_sum[(int64_t)bh * L + row] = (int32_t)sum;

    // Column sums of V over every key the steps below cover (keys up to the end of this query tile
    // under the causal mask, else all): the correction for feeding the probabilities to the signed
    // MFMA as P - 128.  A small kernel ahead of this one left the sums of each BQ-key chunk.
    if (tid < D) {
        const int32_t *cp = p.ws_colsum + (int64_t)(b * p.Hkv + kvh) * p.n_qtiles * D + tid;
        const int nchunk = CAUSAL ? qt + 1 : p.n_qtiles;
        int32_t acc = 0;
#pragma unroll 8
        for (int c = 0; c < nchunk; ++c) acc += cp[(int64_t)c * D];
        colsum[tid] = acc;
    }
    __syncthreads(); // LUT_hat, K(0), V(0), K(1) are in LDS

    // per-row probability table: PT[idx] = round(255 * LUT_hat[idx] / sum) - 128 as a byte
    {
        const uint8_t *lut_b = (const uint8_t *)lut_lds;
        uint32_t *pt = PT[wave];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int kidx = 16 * h + j;
            const uint32_t e = lut_b[kidx];
            const uint32_t pr = (510u * e + sum) / (2u * sum);
            pt[kidx * 32 + n] = (pr ^ 0x80u) & 0xffu;
        }
    }
    const uint32_t *pt = PT[wave] + n;

    // ---- LDS read addresses (lane constants; sub-tile and buffer go into immediate offsets)
    int kf_off[KB], vf_off[CB];
    {
        const int sw = swz_k<D>(n); // equal for keys n and n + 32
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf_off[kb] = n * D + (((2 * kb + h) ^ sw) << 4);
        // transposing read: lanes 2j, 2j+1 of a 16-lane group point at the two 8-byte halves of key
        // row j's 16 channels; lane i of the group receives channel i of the eight rows.
        const int tr_i = lane & 15, tr_g = (lane >> 4) & 1, jj = tr_i >> 1;
        const int key = 8 * (jj >> 2) + 4 * h + (jj & 3); // + 16 for the second half of the operand
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) vf_off[cb] = key * D + (((2 * cb + tr_g) ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
    }
    auto read_kf = [&](const int8_t *Ksub, v4i (&kf)[KB]) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = *(const v4i *)(Ksub + kf_off[kb]);
    };
    auto read_vf = [&](const int8_t *Vsub, v4i (&vf)[CB]) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + vf_off[cb]));
            const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(Vsub + vf_off[cb] + 16 * D));
            vf[cb] = v4i{x0[0], x0[1], x1[0], x1[1]};
        }
    };
    auto visible = [&](int key) { return key < L && (!CAUSAL || key <= row); };

    // ---- pipeline state
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0;
    v4i kf[KB], vf[CB], pf;
    v16i sA, sB;          // raw scores of the sub-tile in flight / being accumulated
    uint32_t lA[16], lB[16]; // looked-up probability bytes (xor 0x80) of a sub-tile

    // packs the looked-up bytes of sub-tile jp into operand register g
    auto pack = [&](auto masked_tag, int jp, const uint32_t (&l)[16], int g) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        uint32_t b4[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            b4[r] = l[4 * g + r];
            if (MASKED) b4[r] = visible(32 * jp + acc_key(4 * g + r, h)) ? b4[r] : 0x80u;
        }
        pf[g] = (int)(((b4[1] << 8) | b4[0]) | (((b4[3] << 8) | b4[2]) << 16));
    };

    // One pipeline step (see the head of the file).  sc: scores of sub-tile j; sn: receives the
    // scores of sub-tile j+1; lp: lookups of sub-tile j-1; lc: receives the lookups of sub-tile j.
    // On entry kf holds the K fragments of sub-tile j+1 and vf the V^T fragments of sub-tile j-1.
    auto step = [&](auto masked_tag, int j, const int8_t *Knext, const int8_t *Vcur, const v16i &sc, v16i &sn,
                    const uint32_t (&lp)[16], uint32_t (&lc)[16]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int sl = 0; sl < NSLOT; ++sl) {
            if (sl == 0) sn = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[0], qf[0], v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0);
            else if (sl < KB) sn = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[sl], qf[sl], sn, 0, 0, 0);
            else o[sl - KB] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[sl - KB], pf, o[sl - KB], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = sl * EPS; e < (sl + 1) * EPS; ++e) {
                // hidden keys may exceed the row max
                const int c = MASKED ? min(max(sc[e], ri.bound), ri.mx) : max(sc[e], ri.bound);
                lc[e] = pt[ri(c) * 32];
            }
            if (sl < KB) {
#pragma unroll
                for (int g = sl * GPS; g < (sl + 1) * GPS; ++g) pack(masked_tag, j - 1, lp, g);
            }
            if (sl == KB - 1) read_kf(Knext, kf); // the scores' MFMAs have all issued
            if (sl == NSLOT - 1) read_vf(Vcur, vf);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One iteration = tile T: its two sub-tiles' lookups, the scores of tile T+1's sub-tiles.
    // PAR = T & 1 names the buffers statically: K(T+1) is in Ks[PAR^1], V(T) in Vs[PAR].
    auto iteration = [&](auto masked_tag, auto par_tag, int T) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        int8_t *Kdma = PAR ? Ks1 : Ks0;             // K(T+2) replaces K(T), consumed an iteration ago
        int8_t *Vdma = PAR ? Vs0 : Vs1;             // V(T+1) replaces V(T-1)
        const int8_t *Krd = PAR ? Ks0 : Ks1;
        const int8_t *Vrd = PAR ? Vs1 : Vs0;
        if (T + 2 < ntiles) dma_k(T + 2, Kdma);
        if (T + 1 < ntiles) dma_v(T + 1, Vdma);
        step(masked_tag, 2 * T, Krd, Vrd, sA, sB, lB, lA);
        step(masked_tag, 2 * T + 1, Krd + SUB, Vrd + SUB, sB, sA, lA, lB);
        __syncthreads();
    };

    // ---- prologue: scores of sub-tile 0, fragments of sub-tile 1; an empty "sub-tile -1"
    read_kf(Ks0, kf);
    sA = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) sA = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[kb], sA, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_kf(Ks0 + SUB, kf);
#pragma unroll
    for (int i = 0; i < 16; ++i) lB[i] = 0; // operand bytes 0 = probability 128 - 128: adds nothing
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) vf[cb] = v4i{0, 0, 0, 0};
    pf = v4i{0, 0, 0, 0};
    __syncthreads(); // every wave has read K(0) before iteration 0 overwrites it with K(2)

    // iterations whose two sub-tiles are fully visible to this wave need no masks (wave-uniform)
    const int nfull_sub = CAUSAL ? min(L / 32, (qw0 + 1) / 32) : L / 32;
    const int nhot = min(nfull_sub / 2, ntiles);
    for (int T = 0; T < ntiles; T += 2) {
        if (T < nhot) iteration(std::false_type{}, std::integral_constant<int, 0>{}, T);
        else iteration(std::true_type{}, std::integral_constant<int, 0>{}, T);
        if (T + 1 < ntiles) {
            if (T + 1 < nhot) iteration(std::false_type{}, std::integral_constant<int, 1>{}, T + 1);
            else iteration(std::true_type{}, std::integral_constant<int, 1>{}, T + 1);
        }
    }
    // ---- drain: the last sub-tile's probabilities meet V (its lookups are in lB, its V^T in vf)
#pragma unroll
    for (int g = 0; g < 4; ++g) pack(std::true_type{}, 2 * ntiles - 1, lB, g);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[cb], pf, o[cb], 0, 0, 0);

    // ================================================================= epilogue (Sec. 3.2: requantization)
    if (row >= L) return;
    int8_t *Op = p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)row * p.os[2];
    const int64_t half = 1ll << (hp.rq_shift - 1);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int ch0 = cb * 32 + 8 * g + 4 * h;
            uint32_t packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int32_t acc = o[cb][4 * g + r] + 128 * colsum[ch0 + r];
                if (p.dbg_acc) p.dbg_acc[((int64_t)bh * L + row) * D + ch0 + r] = acc;
                int64_t v = ((int64_t)acc * hp.rq_mult + half) >> hp.rq_shift;
                v = v > 127 ? 127 : (v < -127 ? -127 : v);
                packed |= ((uint32_t)(int)v & 0xffu) << (8 * r);
            }
            *(uint32_t *)(Op + ch0) = packed;
        }
    }
}

template <int D, bool CAUSAL>
int launch_mode(const FwdParams &p, int idx_mode, hipStream_t st)
{
    const dim3 grid((unsigned)fwd_grid_size(p.B, p.Hq, p.Hkv, p.n_qtiles)), block(NT);
    if (idx_mode == IDX_MAD24)
        hipLaunchKernelGGL((sweep_c_kernel<D, CAUSAL, IDX_MAD24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_MULHI24)
        hipLaunchKernelGGL((sweep_c_kernel<D, CAUSAL, IDX_MULHI24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_FP32)
        hipLaunchKernelGGL((sweep_c_kernel<D, CAUSAL, IDX_FP32>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((sweep_c_kernel<D, CAUSAL, IDX_DIV>), grid, block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// p.n_qtiles must count tiles of 128 query rows; p.ws_row_max / ws_row_sum / ws_colsum filled.
int launch_sweep_c(const FwdParams &p, int d, int idx_mode, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (d == 64) return p.causal ? launch_mode<64, true>(p, idx_mode, st) : launch_mode<64, false>(p, idx_mode, st);
    if (d == 128) return p.causal ? launch_mode<128, true>(p, idx_mode, st) : launch_mode<128, false>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
