// Sweeps A and B of the IntAttention forward as a kernel of its own (gfx950): the exact row maximum
// of the INT8 scores (sweep A), then with it the row sum of E_hat = LUT_hat[idx] (sweep B,
// Sec. 3.1: clip at c_int, index map, table lookup).  Both go to a workspace, 8 bytes per query
// row, for the sweep C kernel.  The scores are recomputed in each sweep instead of ever being stored.
//
// Same data layout and lane ownership as the other forward kernels (transposed scores, one query
// row per lane, XOR-swizzled K tiles in LDS filled by direct global->LDS loads); a wave owns RB
// blocks of 32 query rows, so every K fragment read from LDS feeds RB MFMAs.  The key axis is
// walked in steps of 32 keys as a software pipeline inside each wave: step j issues
//     one MFMA of the scores of sub-tile j+1, then the vector work of EPS scores of sub-tile j,
//     one MFMA, ...
// and each K fragment register is refilled (sub-tile j+2) right after its last MFMA of the step has
// issued.  In sweep B a looked-up table entry is added to the row sum half a step after its lookup
// was issued, so nothing waits on what it has just issued.  Scheduling barriers pin that order.
//
// Tiles are 64 keys (two steps), double buffered, one barrier per tile: iteration T reads K tile
// T+1 and, at its top, requests K tile T+2 into the buffer that was read an iteration ago.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;

template <int D, int RB, bool CAUSAL, int MODE>
__global__ __launch_bounds__(NT, RB == 1 ? 3 : 2) void sweep_ab_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;       // 32-wide blocks of the head dimension
    constexpr int NSUB = 2;          // sub-tiles (pipeline steps) per tile
    constexpr int BK = 32 * NSUB;    // keys per tile
    constexpr int BQ = WAVES * RB * 32;
    constexpr int TILE = BK * D;     // bytes
    constexpr int SUB = 32 * D;      // bytes of a 32-key sub-tile
    constexpr int NBLK = TILE / 1024;
    constexpr int JB = (NBLK + WAVES - 1) / WAVES;
    constexpr int CPR = D / 16;
    constexpr int RPB = 1024 / D;
    constexpr int NSLOT = RB * KB;        // MFMAs per step
    constexpr int NEL = 16 * RB;          // scores per lane and step
    constexpr int EPS = NEL / NSLOT;      // scores handled after each MFMA
    constexpr int HALF = NSLOT / 2;
    static_assert(NEL % NSLOT == 0 && NSLOT % 2 == 0, "vector work must split evenly over the MFMA slots");

    __shared__ __attribute__((aligned(1024))) int8_t Ks0[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Ks1[TILE];
    __shared__ uint32_t lut_lds[8];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return; // padding of the XCD-aware grid (uniform for the whole workgroup)
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt + p.row_lo / BQ;
    const int bh = b * p.Hq + hq;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    if (p.filter && hp.pad[0] != MODE) return; // another launch of this pair serves the head (uniform for the workgroup)
    const int L = p.Lk; // keys
    // query rows: [rlo, rhi) of the numbering in which row r sees keys <= r under the causal mask
    const int rlo = p.row_lo, rhi = p.row_lo + p.L, LQ = p.L;
    // parameters of the block of query rows that `row` lies in (finer groups over query rows, Sec. 3.3)
    auto row_hp = [&](int row) __attribute__((always_inline)) {
        const int lr = (row >= rlo && row < rhi) ? row - rlo : 0;
        return p.row_table[(int64_t)bh * p.n_rowblk + lr / p.q_block];
    };
    const uint32_t top = (uint32_t)p.top;

    const int q0 = qt * BQ, qw0 = q0 + wave * (RB * 32);
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];

    if (tid < 8) lut_lds[tid] = p.lut[tid];

    // Q fragments: row block rb, row qw0 + 32 rb + n, bytes [32 kb + 16 h, +16)
    v4i qf[RB][KB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = qw0 + 32 * rb + n;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            qf[rb][kb] = v4i{0, 0, 0, 0};
            if (row >= rlo && row < rhi) qf[rb][kb] = *(const v4i *)(Qp + (int64_t)(row - rlo) * p.qs[2] + kb * 32 + h * 16);
        }
    }

    const int kmax = CAUSAL ? min(L, q0 + BQ) : L;
    const int ntiles = (kmax + BK - 1) / BK;

    // ---- staging: direct global -> LDS loads; the XOR swizzle is applied to the global address
    // (lane i of a wave-wide 16-byte load lands at byte 16 i of its 1 KiB block).  The loads go
    // through a buffer descriptor that starts at the tile and ends with the last byte of key row
    // L-1, so key rows at or past L come back as zeros from the range check.
    int dma_goff_k[JB];
#pragma unroll
    for (int j = 0; j < JB; ++j) {
        const int key = (wave + WAVES * j) * RPB + lane / CPR, cp = lane % CPR;
        dma_goff_k[j] = key * (int)p.ks[2] + ((cp ^ swz_k<D>(key)) << 4); // the host checked BK * stride < 2^31
    }
    auto dma_k = [&](int t, int8_t *dst) __attribute__((always_inline)) {
        const int8_t *tb = Kp + (int64_t)t * BK * p.ks[2]; // wave-uniform
        const int64_t rem = (int64_t)(L - t * BK - 1) * p.ks[2] + D;
        const uint32_t nrec = rem <= 0 ? 0u : (rem > 0xffffffffll ? 0xffffffffu : (uint32_t)rem); // 0: all of it past L
#if defined(__HIP_DEVICE_COMPILE__) // the host pass has neither the descriptor type nor the builtins
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)tb, 0, (int)nrec, 0x00020000);
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int blk = wave + WAVES * j;
            if (NBLK % WAVES != 0 && blk >= NBLK) continue; // wave-uniform
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(dst + blk * 1024), 16,
                                                     dma_goff_k[j], 0, 0, 0);
        }
#else
        (void)tb, (void)nrec, (void)dst;
#endif
    };

    // ---- LDS read addresses of the K fragments (lane constants)
    int kf_off[KB];
    {
        const int sw = swz_k<D>(n); // equal for keys n and n + 32
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf_off[kb] = n * D + (((2 * kb + h) ^ sw) << 4);
    }
    auto visible = [&](int key, int rb) { return key < L && (!CAUSAL || key <= qw0 + 32 * rb + n); };

    // ---- pipeline state
    v4i kf[KB];
    v16i sA[RB], sB[RB];       // raw scores of the sub-tile in flight / being accumulated
    uint32_t lA[NEL], lB[NEL]; // sweep B: looked-up table entries; only half a step's worth is live
    int mx[RB];
    uint32_t sum[RB];
    RowIndex<MODE> ri[RB];
    const uint8_t *lut_b = (const uint8_t *)lut_lds;

    // One pipeline step.  sc: scores of sub-tile j; sn: receives the scores of sub-tile j+1 (its K
    // fragments are in kf on entry; kf leaves holding those of sub-tile j+2, read from Knext).
    // Sweep B: lc receives the lookups of sub-tile j, lp holds those of sub-tile j-1.
    auto step = [&](auto sweep_tag, auto masked_tag, int j, const int8_t *Knext, const v16i (&sc)[RB], v16i (&sn)[RB],
                    const uint32_t (&lp)[NEL], uint32_t (&lc)[NEL]) __attribute__((always_inline)) {
        constexpr int SW = decltype(sweep_tag)::value;
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int sl = 0; sl < NSLOT; ++sl) {
            const int kb = sl / RB, rbm = sl % RB;
            if (kb == 0)
                sn[rbm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[0], qf[rbm][0], v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0);
            else
                sn[rbm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[rbm][kb], sn[rbm], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (rbm == RB - 1) kf[kb] = *(const v4i *)(Knext + kf_off[kb]); // its last MFMA of this step has issued
            if (SW == 0) {
#pragma unroll
                for (int w = sl * EPS; w < (sl + 1) * EPS; w += 2) {
                    const int rb = w / 16, e = w % 16;
                    if (MASKED) {
                        mx[rb] = visible(32 * j + acc_key(e, h), rb) ? max(mx[rb], sc[rb][e]) : mx[rb];
                        mx[rb] = visible(32 * j + acc_key(e + 1, h), rb) ? max(mx[rb], sc[rb][e + 1]) : mx[rb];
                    } else {
                        mx[rb] = max(max(sc[rb][e], sc[rb][e + 1]), mx[rb]);
                    }
                }
            } else {
                // add what was looked up half a step ago
#pragma unroll
                for (int w = sl * EPS; w < (sl + 1) * EPS; ++w) {
                    const int wp = sl < HALF ? w + HALF * EPS : w - HALF * EPS;
                    const int jp = sl < HALF ? j - 1 : j;
                    const int rb = wp / 16, e = wp % 16;
                    uint32_t l = sl < HALF ? lp[wp] : lc[wp];
                    if (MASKED) l = visible(32 * jp + acc_key(e, h), rb) ? l : 0u;
                    sum[rb] += l;
                }
#pragma unroll
                for (int w = sl * EPS; w < (sl + 1) * EPS; ++w) {
                    const int rb = w / 16, e = w % 16;
                    // hidden keys may exceed the row max
                    const int c = MASKED ? min(max(sc[rb][e], ri[rb].bound), ri[rb].mx) : max(sc[rb][e], ri[rb].bound);
                    lc[w] = lut_b[ri[rb](c)];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One iteration = tile T: the vector work of its two sub-tiles, the scores of the two after them.
    // K tile T+2 replaces K tile T (read an iteration ago) in Kdma; K tile T+1 is read from Krd.
    auto iteration = [&](auto sweep_tag, auto masked_tag, int T, int8_t *Kdma, const int8_t *Krd) __attribute__((always_inline)) {
        if (T + 2 < ntiles) dma_k(T + 2, Kdma);
        step(sweep_tag, masked_tag, 2 * T, Krd, sA, sB, lB, lA);
        step(sweep_tag, masked_tag, 2 * T + 1, Krd + SUB, sB, sA, lA, lB);
        __syncthreads();
    };

    // iterations whose sub-tiles are all fully visible to this wave need no masks (wave-uniform)
    const int nfull_sub = CAUSAL ? min(L / 32, (qw0 + 1) / 32) : L / 32;
    const int nhot = min(nfull_sub / NSUB, ntiles);

    // One sweep over the keys.  The unmasked iterations run in pairs in a loop of their own, every
    // buffer named statically and no branch inside the body; the few remaining ones take the masked
    // code with the buffers chosen at run time.
    auto sweep = [&](auto sweep_tag) __attribute__((always_inline)) {
        dma_k(0, Ks0);
        if (ntiles > 1) dma_k(1, Ks1);
        __syncthreads(); // K tiles 0 and 1 (and LUT_hat) are in LDS
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = *(const v4i *)(Ks0 + kf_off[kb]);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            sA[rb] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) sA[rb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[rb][kb], sA[rb], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = *(const v4i *)(Ks0 + SUB + kf_off[kb]);
#pragma unroll
        for (int i = 0; i < NEL; ++i) lB[i] = 0; // an empty "sub-tile -1"
        __syncthreads(); // every wave has read K tile 0 before iteration 0 overwrites it with K tile 2
        int T = 0;
        for (; T + 2 <= nhot; T += 2) {
            iteration(sweep_tag, std::false_type{}, T, Ks0, Ks1);
            iteration(sweep_tag, std::false_type{}, T + 1, Ks1, Ks0);
        }
#pragma unroll 1
        for (; T < ntiles; ++T) {
            const bool odd = T & 1;
            iteration(sweep_tag, std::true_type{}, T, odd ? Ks1 : Ks0, odd ? Ks0 : Ks1);
        }
    };

    // ================================================================= sweep A: row max
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) mx[rb] = INT32_MIN;
    sweep(std::integral_constant<int, 0>{});
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        mx[rb] = max(mx[rb], __shfl_xor(mx[rb], 32));
        ri[rb].init(MODE == IDX_ROW64 ? row_hp(qw0 + 32 * rb + n) : hp, mx[rb], top);
        sum[rb] = 0;
    }

    // ================================================================= sweep B: row sum of E_hat
    sweep(std::integral_constant<int, 1>{});
    // the second half of the last sub-tile's lookups is still to be added
#pragma unroll
    for (int w = HALF * EPS; w < NEL; ++w) {
        const int rb = w / 16, e = w % 16;
        sum[rb] += visible(32 * (NSUB * ntiles - 1) + acc_key(e, h), rb) ? lB[w] : 0u;
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        sum[rb] += __shfl_xor(sum[rb], 32);
        const int row = qw0 + 32 * rb + n;
        if (h == 0 && row >= rlo && row < rhi) {
            p.ws_row_max[(int64_t)bh * LQ + (row - rlo)] = mx[rb];
            p.ws_row_sum[(int64_t)bh * LQ + (row - rlo)] = (int32_t)sum[rb];
        }
    }
}

template <int D, int RB, bool CAUSAL>
int launch_mode(const FwdParams &p, int idx_mode, hipStream_t st)
{
    const dim3 grid((unsigned)fwd_grid_size(p.B, p.Hq, p.Hkv, p.n_qtiles)), block(NT);
    if (idx_mode == IDX_DEVICE) {
        // the scheme of each head is known on the device only: one launch per scheme, each
        // skipping the heads of the other
        FwdParams pf = p;
        pf.filter = 1;
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_FP32>), grid, block, 0, st, pf);
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_FP64>), grid, block, 0, st, pf);
        return (int)hipGetLastError();
    }
    if (idx_mode == IDX_MAD24)
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_MAD24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_MULHI24)
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_MULHI24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_FP32)
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_FP32>), grid, block, 0, st, p);
    else if (idx_mode == IDX_ROW64)
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_ROW64>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((sweep_ab_kernel<D, RB, CAUSAL, IDX_FP64>), grid, block, 0, st, p);
    return (int)hipGetLastError();
}

template <int RB>
int launch_rb(const FwdParams &p, int d, int idx_mode, hipStream_t st)
{
    if (d == 64) return p.causal ? launch_mode<64, RB, true>(p, idx_mode, st) : launch_mode<64, RB, false>(p, idx_mode, st);
    if (d == 128) return p.causal ? launch_mode<128, RB, true>(p, idx_mode, st) : launch_mode<128, RB, false>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace

// rows_per_wave is 32 or 64; p.n_qtiles must count tiles of 4 * rows_per_wave query rows;
// p.ws_row_max / ws_row_sum receive the results.
int launch_sweep_ab(const FwdParams &p, int d, int idx_mode, int rows_per_wave, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (rows_per_wave == 32) return launch_rb<1>(p, d, idx_mode, st);
    if (rows_per_wave == 64) return launch_rb<2>(p, d, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
