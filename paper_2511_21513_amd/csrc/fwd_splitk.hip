// Fused IntAttention forward for mid-size problems on gfx950 (MI355X): one workgroup per block of 32
// query rows, the KEYS of that block split over the four waves of the workgroup.
//
// With 128-row tiles a problem of a few hundred workgroups leaves most SIMDs with one wave that walks
// every key of its tile three times; the longest tile sets the time.  Here every wave takes every
// fourth 32-key sub-tile of the block's keys (interleaved, so the causal triangle is shared evenly),
// so the longest chain is a quarter as long and there are four times as many workgroups.  The three
// reductions of IndexSoftmax (Sec. 3.1-3.2: row max, row sum of E_hat, P_hat.V_hat) cross the waves
// through LDS once each:
//   sweep A: S^T = K.Q^T of the wave's sub-tiles -> row max -> max over the waves
//   sweep B: S^T again -> clip, index, LUT_hat -> row sum -> sum over the waves -> per-row table
//            P_hat = round(255 E/S) (Eq. uint8-prob), built once per workgroup
//   sweep C: S^T again -> index -> table -> 16 probability bytes per lane = one MFMA B operand of
//            O^T += V^T.P^T -> accumulators added up over the waves in LDS -> requantize, store.
// A wave works alone between the reductions: K fragments come straight from global memory (a lane reads
// the 16 bytes of its key row that its MFMA operand holds; the next sub-tile is requested before this one is
// computed), V sub-tiles go through a wave-private LDS buffer (direct global -> LDS loads, then the
// transposing LDS read), and there is no workgroup barrier inside a sweep.
//
// Probabilities go to the signed MFMA as P - 128; the correction, 128 * (column sums of V over every key of
// the processed sub-tiles), comes from one more MFMA per channel block and sub-tile against an operand of
// all ones, which leaves the column sums in the accumulator layout of the outputs: one launch, no workspace.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;

template <int D, bool CAUSAL, int MODE>
__global__ __launch_bounds__(NT, D == 64 ? 4 : 2) void fwd_splitk_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;  // 32-wide blocks of the head dimension
    constexpr int CB = D / 32;  // 32-wide blocks of output channels
    constexpr int SUB = 32 * D; // bytes of a 32-key sub-tile
    [[maybe_unused]] constexpr int NBLK = SUB / 1024; // 1 KiB blocks of a sub-tile: one wave-wide 16-byte load each
    [[maybe_unused]] constexpr int CPR = D / 16;      // 16-byte chunks per key row
    [[maybe_unused]] constexpr int RPB = 1024 / D;    // key rows per block

    // wave-private V sub-tiles, two buffers as separate arrays (the compiler tracks each direct-to-LDS load by
    // the array it targets, so reads of one buffer need not wait for loads into the other)
    __shared__ __attribute__((aligned(1024))) int8_t Vw0[WAVES][SUB];
    __shared__ __attribute__((aligned(1024))) int8_t Vw1[WAVES][SUB];
    __shared__ int32_t acc_lds[32][D + 1]; // output accumulators, summed over the waves (rows padded: one bank per row)
    __shared__ int32_t red[2][WAVES][32];                               // per-wave row max / row sum
    __shared__ uint32_t lut_lds[16];
    extern __shared__ uint32_t PT[]; // [idx][row], NIDX * 32 words

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return; // padding of the XCD-aware grid (uniform for the whole workgroup)
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt + p.row_lo / 32;
    const int bh = b * p.Hq + hq;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    if (p.filter && (hp.pad[0] == IDX_TOP24 ? (int)IDX_MAD24 : hp.pad[0]) != MODE) return; // served by the other launch
    const int L = p.Lk;
    const int rlo = p.row_lo, rhi = p.row_lo + p.L, LQ = p.L;
    const uint32_t top = (uint32_t)p.top;
    const int NIDX = top < 32 ? 32 : 64;

    const int q0 = qt * 32, row = q0 + n; // the lane's query row (numbering in which row r sees keys <= r)
    const bool row_ok = row >= rlo && row < rhi;
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    if (tid < 16) lut_lds[tid] = p.lut[tid];
    for (int i = tid; i < 32 * (D + 1); i += NT) (&acc_lds[0][0])[i] = 0;

    // Q fragments: row q0 + n, bytes [32 kb + 16 h, +16)
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (row_ok) qf[kb] = *(const v4i *)(Qp + (int64_t)(row - rlo) * p.qs[2] + kb * 32 + h * 16);
    }

    const int kmax = CAUSAL ? min(L, q0 + 32) : L; // keys any row of the block sees
    const int nsub = (kmax + 31) / 32;             // sub-tiles of the block; wave w takes w, w + 4, ...

    // K fragments of sub-tile j straight from global memory: key row 32 j + n, bytes [32 kb + 16 h, +16)
    auto load_kf = [&](int j, v4i (&kf)[KB]) __attribute__((always_inline)) {
        // key rows at or past L: the last row is read instead; their scores are hidden keys and never used
        const int key = min(32 * j + n, L - 1);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) kf[kb] = v4i{0, 0, 0, 0};
        if (j < nsub) { // wave-uniform
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) kf[kb] = *(const v4i *)(Kp + (int64_t)key * p.ks[2] + kb * 32 + h * 16);
        }
    };
    auto scores = [&](const v4i (&kf)[KB]) __attribute__((always_inline)) {
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[kb], s, 0, 0, 0);
        return s;
    };
    auto visible = [&](int key) { return key < L && (!CAUSAL || key <= row); };
    // wave-uniform: every key of sub-tile j is visible to every row of the block
    auto sub_is_full = [&](int j) { return 32 * j + 32 <= L && (!CAUSAL || 32 * j + 31 <= q0); };

    // The wave's sub-tiles in order, K fragments of the next one requested before this one is computed; the two
    // register sets (and V buffers) alternate statically, so nothing is copied and no wait is forced early.
    // body(j, kf, buffer number); prefetch(j, buffer number) is called with the K request of sub-tile j.
    auto walk = [&](auto prefetch, auto body) __attribute__((always_inline)) {
        v4i kA[KB], kB[KB];
        load_kf(wave, kA);
        prefetch(wave, 0);
        for (int j = wave; j < nsub; j += 2 * WAVES) {
            load_kf(j + WAVES, kB);
            prefetch(j + WAVES, 1);
            body(j, kA, 0);
            if (j + WAVES < nsub) {
                load_kf(j + 2 * WAVES, kA);
                prefetch(j + 2 * WAVES, 0);
                body(j + WAVES, kB, 1);
            }
        }
    };
    auto no_prefetch = [&](int, int) {};

    // ================================================================= sweep A: row max
    int mx = INT32_MIN;
    walk(no_prefetch, [&](int j, const v4i (&kf)[KB], int) __attribute__((always_inline)) {
        const v16i s = scores(kf);
        if (sub_is_full(j)) {
#pragma unroll
            for (int i = 0; i < 16; i += 2) mx = max(max(s[i], s[i + 1]), mx);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = visible(32 * j + acc_key(i, h)) ? max(mx, s[i]) : mx;
        }
    });
    mx = max(mx, __shfl_xor(mx, 32));
    if (h == 0) red[0][wave][n] = mx;
    __syncthreads(); // (also: lut_lds and the zeroed accumulators are visible)
    mx = max(max(red[0][0][n], red[0][1][n]), max(red[0][2][n], red[0][3][n]));
    if (!row_ok) mx = 0; // rows outside the problem: zero scores, never stored

    RowIndex<MODE> ri;
    ri.init(hp, mx, top);

    // ================================================================= sweep B: row sum of E_hat
    const uint8_t *lut_b = (const uint8_t *)lut_lds;
    uint32_t sum = 0;
    walk(no_prefetch, [&](int j, const v4i (&kf)[KB], int) __attribute__((always_inline)) {
        const v16i s = scores(kf);
        if (sub_is_full(j)) {
            uint32_t e[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) e[i] = lut_b[ri(max(s[i], ri.bound))];
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += e[i];
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t e = lut_b[ri(min(max(s[i], ri.bound), ri.mx))]; // hidden keys may exceed the row max
                sum += visible(32 * j + acc_key(i, h)) ? e : 0u;
            }
        }
    });
    sum += __shfl_xor(sum, 32);
    if (h == 0) red[1][wave][n] = (int32_t)sum;
    __syncthreads();
    sum = (uint32_t)red[1][0][n] + (uint32_t)red[1][1][n] + (uint32_t)red[1][2][n] + (uint32_t)red[1][3][n];
    if (sum == 0) sum = 1; // only rows outside [rlo, rhi); never stored
    if (wave == 0 && h == 0 && row_ok) {
        if (p.dbg_row_max) p.dbg_row_max[(int64_t)bh * LQ + (row - rlo)] = mx;
        if (p.dbg_row_sum) p.dbg_row_sum[(int64_t)bh * LQ + (row - rlo)] = (int32_t)sum;
    }
    // per-row probability table, once per workgroup: PT[idx][row] = round(255 LUT_hat[idx] / S) - 128 as a byte
    for (int e = tid; e < NIDX * 32; e += NT) {
        const int idx = e >> 5, r = e & 31;
        const uint32_t S = (uint32_t)red[1][0][r] + (uint32_t)red[1][1][r] + (uint32_t)red[1][2][r] + (uint32_t)red[1][3][r];
        const uint32_t Sd = S ? S : 1u;
        const uint32_t ev = (uint32_t)idx <= top ? lut_b[idx] : 0u;
        PT[e] = (prob_u8(ev, Sd, __builtin_amdgcn_rcpf((float)(2u * Sd))) ^ 0x80u) & 0xffu;
    }
    __syncthreads();

    // ================================================================= sweep C: P_hat and P_hat.V_hat
    // V sub-tile j into this wave's buffer `buf`: direct global -> LDS loads, the XOR swizzle applied to the
    // global address; rows at or past L arrive as zeros from the range check of the buffer descriptor
    auto stage_v = [&](int j, int buf) __attribute__((always_inline)) {
        if (j >= nsub) return; // wave-uniform
        const int key0 = 32 * j;
        const int8_t *tb = Vp + (int64_t)key0 * p.vs[2];
        const int64_t rem = (int64_t)(L - key0 - 1) * p.vs[2] + D;
        const uint32_t nrec = rem <= 0 ? 0u : (rem > 0xffffffffll ? 0xffffffffu : (uint32_t)rem);
#if defined(__HIP_DEVICE_COMPILE__) // the host pass has neither the descriptor type nor the builtins
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)tb, 0, (int)nrec, 0x00020000);
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            const int key = blk * RPB + lane / CPR, cpos = lane % CPR;
            const int goff = key * (int)p.vs[2] + ((cpos ^ swz_v<D>(key)) << 4); // the host checked 128 * stride < 2^31
            int8_t *dst = (buf ? &Vw1[wave][0] : &Vw0[wave][0]) + blk * 1024;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)dst, 16, goff, 0, 0, 0);
        }
#else
        (void)tb, (void)nrec, (void)buf;
#endif
    };
    // transposing read of V^T fragments: lanes 2j, 2j+1 of a 16-lane group point at the two 8-byte halves of a key row
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1;
    auto vt_frag = [&](const int8_t *Vb, int cb) __attribute__((always_inline)) {
        v4i a;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int jj = tr_i >> 1;
            const int key = 8 * (2 * r + (jj >> 2)) + 4 * h + (jj & 3);
            const int c16 = 2 * cb + tr_g;
            const int8_t *ptr = Vb + key * D + ((c16 ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
            const v2i x = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)ptr);
            a[2 * r] = x[0];
            a[2 * r + 1] = x[1];
        }
        return a;
    };

    v16i o[CB], ocs[CB]; // P_hat.V_hat with P - 128, and the column sums of V over the same keys
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0, ocs[cb][i] = 0;
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const uint32_t *pt = PT + n;
    walk(stage_v, [&](int j, const v4i (&kf)[KB], int buf) __attribute__((always_inline)) {
        v16i s = scores(kf);
        const bool full = sub_is_full(j);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int sc = full ? max(s[i], ri.bound) : min(max(s[i], ri.bound), ri.mx);
            s[i] = (int)pt[ri(sc) * 32];
        }
        v4i pf;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t pb4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 4 * g + r;
                pb4[r] = (uint32_t)s[i];
                if (!full) pb4[r] = visible(32 * j + acc_key(i, h)) ? pb4[r] : 0x80u;
            }
            pf[g] = (int)(((pb4[1] << 8) | pb4[0]) | (((pb4[3] << 8) | pb4[2]) << 16));
        }
        // (the compiler waits for this wave's direct-to-LDS loads into the buffer before the reads below)
        const int8_t *Vb = buf ? &Vw1[wave][0] : &Vw0[wave][0];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const v4i vf = vt_frag(Vb, cb);
            o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, o[cb], 0, 0, 0);
            ocs[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, ones, ocs[cb], 0, 0, 0);
        }
    });
    // the accumulators of the four waves meet in LDS: register i of lane (n, h) in channel block cb is
    // row n, channel 32 cb + 8 (i / 4) + 4 h + (i % 4)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) atomicAdd(&acc_lds[n][cb * 32 + 8 * (i >> 2) + 4 * h + (i & 3)], o[cb][i] + 128 * ocs[cb][i]);
    __syncthreads();

    // ================================================================= epilogue: 8 threads per row
    constexpr int CPT = D / 8; // channels per thread
    const int er = tid >> 3, ec0 = (tid & 7) * CPT, erow = q0 + er;
    if (erow >= rlo && erow < rhi) {
        int8_t *Op = p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)(erow - rlo) * p.os[2];
#pragma unroll
        for (int c4 = 0; c4 < CPT; c4 += 4) {
            uint32_t packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ch = ec0 + c4 + r;
                const int32_t acc = acc_lds[er][ch];
                if (p.dbg_acc) p.dbg_acc[((int64_t)bh * LQ + (erow - rlo)) * D + ch] = acc;
                packed |= ((uint32_t)requant_any(acc, hp.rq_mult, hp.rq_shift) & 0xffu) << (8 * r);
            }
            *(uint32_t *)(Op + ec0 + c4) = packed;
        }
    }
}

template <int D, bool CAUSAL>
int launch_mode(const FwdParams &p, int idx_mode, hipStream_t st)
{
    const dim3 grid((unsigned)fwd_grid_size(p.B, p.Hq, p.Hkv, p.n_qtiles)), block(NT);
    const unsigned sh = (unsigned)((p.top < 32 ? 32 : 64) * 32 * sizeof(uint32_t)); // the per-row probability table
    if (idx_mode == IDX_DEVICE) {
        FwdParams pf = p;
        pf.filter = 1;
        hipLaunchKernelGGL((fwd_splitk_kernel<D, CAUSAL, IDX_MAD24>), grid, block, sh, st, pf);
        hipLaunchKernelGGL((fwd_splitk_kernel<D, CAUSAL, IDX_FP64>), grid, block, sh, st, pf);
        return (int)hipGetLastError();
    }
    if (idx_mode == IDX_MAD24 || idx_mode == IDX_TOP24) // the top-byte scheme is the multiply-add with the shift at 24
        hipLaunchKernelGGL((fwd_splitk_kernel<D, CAUSAL, IDX_MAD24>), grid, block, sh, st, p);
    else if (idx_mode == IDX_MULHI24)
        hipLaunchKernelGGL((fwd_splitk_kernel<D, CAUSAL, IDX_MULHI24>), grid, block, sh, st, p);
    else if (idx_mode == IDX_FP32)
        hipLaunchKernelGGL((fwd_splitk_kernel<D, CAUSAL, IDX_FP32>), grid, block, sh, st, p);
    else if (idx_mode == IDX_FP64)
        hipLaunchKernelGGL((fwd_splitk_kernel<D, CAUSAL, IDX_FP64>), grid, block, sh, st, p);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

} // namespace

// p.n_qtiles counts 32-row blocks; per-tensor and per-head parameters only (hp0 / hp_table); no workspace.
int launch_fwd_splitk(const FwdParams &p, int d, int idx_mode, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (d == 64) return p.causal ? launch_mode<64, true>(p, idx_mode, st) : launch_mode<64, false>(p, idx_mode, st);
    if (d == 128) return p.causal ? launch_mode<128, true>(p, idx_mode, st) : launch_mode<128, false>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
