// Fused IntAttention forward for gfx950 (MI355X), software-pipelined variant.
//
// Same mathematics and data layout as fwd_kernel.hip (three sweeps over the key axis: row
// max, row sum of E_hat, then P_hat and P_hat.V_hat; Sec. 3.1-3.2), for 32 query rows per
// wave and 64-key LDS tiles.  The difference is the instruction schedule of the two
// ALU-heavy sweeps: the element-wise IndexSoftmax work on one 32x32 score block is issued
// together with the MFMAs that produce the NEXT score block (and, in the last sweep, the
// P_hat.V_hat MFMAs of the PREVIOUS block), so that the matrix core and the vector ALU of
// a SIMD run at the same time from one wave.  Score blocks alternate between two register
// sets.  Because work on a tile now extends past the barrier that publishes the next tile,
// LDS tiles rotate through three buffers instead of two.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;
constexpr int BQ = WAVES * 32;
constexpr int BK = 64;
constexpr int NBUF = 3;

// Compile-time profiling switch: bit 0/1/2 = run sweep A/B/C.  Anything but 7 gives wrong
// results and exists only to time the sweeps separately.
#ifndef INTATTN_PROFILE_SWEEPS
#define INTATTN_PROFILE_SWEEPS 7
#endif

template <int D, bool CAUSAL, int MODE>
__global__ __launch_bounds__(NT, 2) void fwd_pipe_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;
    constexpr int CB = D / 32;
    constexpr int TILE = BK * D;
    constexpr int NCHUNK = TILE / 16;
    constexpr int CPT = NCHUNK / NT;
    static_assert(CPT >= 1 && CPT * NT == NCHUNK, "tile must split evenly over the threads");
    static_assert(CB <= WAVES, "one wave per channel block accumulates the V column sums");

    // One LDS object with the small tables first: their addresses then fit the 16-bit immediate
    // offset of the LDS instructions, which saves an address addition per table lookup.
    struct Smem {
        uint8_t lut[32];
        int32_t colsum[D];
        uint32_t PT[WAVES][32 * 32]; // [idx][row] per wave
        __attribute__((aligned(16))) int8_t Ks[NBUF][TILE];
        __attribute__((aligned(16))) int8_t Vs[NBUF][TILE];
    };
    __shared__ __attribute__((aligned(16))) Smem sm;
    auto &Ks = sm.Ks;
    auto &Vs = sm.Vs;
    auto &PT = sm.PT;
    auto &lut_lds = sm.lut;
    auto &colsum = sm.colsum;

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return; // padding of the XCD-aware grid (uniform for the whole workgroup)
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt;
    const int bh = b * p.Hq + hq;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    const int L = p.L;
    const uint32_t top = (uint32_t)p.top;

    const int q0 = qt * BQ, qw0 = q0 + wave * 32, row = qw0 + n;
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    if (tid < 8) ((uint32_t *)lut_lds)[tid] = p.lut[tid];

    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (row < L) qf[kb] = *(const v4i *)(Qp + (int64_t)row * p.qs[2] + kb * 32 + h * 16);
    }

    const int kmax = CAUSAL ? min(L, q0 + BQ) : L;
    const int ntiles = (kmax + BK - 1) / BK;
    // tiles [0, nfull) are wholly visible to all 32 rows of this wave and need no masks
    const int nfull = min(ntiles, CAUSAL ? min(L, qw0 + 1) / BK : L / BK);

    // ---- staging: global -> registers -> swizzled LDS (see fwd_kernel.hip for the layout)
    v4i stage_k[CPT], stage_v[CPT];
    int st_key[CPT], st_goff_k[CPT], st_goff_v[CPT], st_lds_k[CPT], st_lds_v[CPT];
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
        const int c = tid + j * NT;
        const int key = c / (D / 16), c16 = c % (D / 16);
        st_key[j] = key;
        st_goff_k[j] = key * (int)p.ks[2] + c16 * 16;
        st_goff_v[j] = key * (int)p.vs[2] + c16 * 16;
        st_lds_k[j] = key * D + ((c16 ^ swz_k<D>(key)) << 4);
        st_lds_v[j] = key * D + ((c16 ^ swz_v<D>(key)) << 4);
    }
    auto load_tile = [&](const int8_t *base, int64_t stride, const int (&goff)[CPT], int t, v4i (&st)[CPT]) {
        const int8_t *tb = base + (int64_t)t * BK * stride; // wave-uniform
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const uint32_t off = (t * BK + st_key[j] < L) ? (uint32_t)goff[j] : 0u; // row t*BK exists
            st[j] = *(const v4i *)(tb + off);
        }
    };
    auto store_tile = [&](int8_t *dst, const int (&loff)[CPT], int t, v4i (&st)[CPT]) {
        if ((t + 1) * BK > L) { // wave-uniform: only the last tile can be ragged
#pragma unroll
            for (int j = 0; j < CPT; ++j)
                if (t * BK + st_key[j] >= L) st[j] = v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < CPT; ++j) *(v4i *)(dst + loff[j]) = st[j];
    };
    auto load_k = [&](int t) { load_tile(Kp, p.ks[2], st_goff_k, t, stage_k); };
    auto load_v = [&](int t) { load_tile(Vp, p.vs[2], st_goff_v, t, stage_v); };
    auto store_k = [&](int t) { store_tile(Ks[t % NBUF], st_lds_k, t, stage_k); };
    auto store_v = [&](int t) { store_tile(Vs[t % NBUF], st_lds_v, t, stage_v); };

    // ---- one 32-key x 32-row score block: KB chained MFMAs starting from `s`
    auto qk = [&](const int8_t *kbuf, int st, v16i s) {
        const int key = 32 * st + n;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const v4i a = *(const v4i *)(kbuf + key * D + (((2 * kb + h) ^ swz_k<D>(key)) << 4));
            s = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qf[kb], s, 0, 0, 0);
        }
        return s;
    };
    auto visible = [&](int key) { return key < L && (!CAUSAL || key <= row); };
    // wave-uniform: all 32 keys from klo on are visible to all 32 rows of this wave
    auto block_full = [&](int klo) { return klo + 32 <= L && (!CAUSAL || klo + 31 <= qw0); };

    // transposing read of a V^T fragment (see fwd_kernel.hip)
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1;
    auto vt_frag = [&](const int8_t *vbuf, int st, int cb) {
        v4i a;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int j = tr_i >> 1;
            const int key = 32 * st + 8 * (2 * r + (j >> 2)) + 4 * h + (j & 3);
            const int c16 = 2 * cb + tr_g;
            const int8_t *ptr = vbuf + key * D + ((c16 ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
            const v2i x = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)ptr);
            a[2 * r] = x[0];
            a[2 * r + 1] = x[1];
        }
        return a;
    };

    const v16i zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    // ================================================================= sweep A: row max
    int mx = INT32_MIN;
    load_k(0);
    store_k(0);
    if (ntiles > 1) load_k(1);
    __syncthreads();
    for (int t = 0; t < ((INTATTN_PROFILE_SWEEPS & 1) ? ntiles : 0); ++t) {
        const int8_t *kb_ = Ks[t % NBUF];
        if (!(CAUSAL && t * BK > qw0 + 31)) { // tile not wholly hidden from this wave
            v16i s0 = zero16, s1 = zero16;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) { // two interleaved chains
                const v4i a0 = *(const v4i *)(kb_ + n * D + (((2 * kb + h) ^ swz_k<D>(n)) << 4));
                const v4i a1 = *(const v4i *)(kb_ + (32 + n) * D + (((2 * kb + h) ^ swz_k<D>(32 + n)) << 4));
                s0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, qf[kb], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, qf[kb], s1, 0, 0, 0);
            }
            if (block_full(t * BK + 32)) {
#pragma unroll
                for (int i = 0; i < 16; i += 2) mx = max(max(s0[i], s0[i + 1]), mx);
#pragma unroll
                for (int i = 0; i < 16; i += 2) mx = max(max(s1[i], s1[i + 1]), mx);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    mx = visible(t * BK + acc_key(i, h)) ? max(mx, s0[i]) : mx;
                    mx = visible(t * BK + 32 + acc_key(i, h)) ? max(mx, s1[i]) : mx;
                }
            }
        }
        if (t + 1 < ntiles) store_k(t + 1);
        if (t + 2 < ntiles) load_k(t + 2);
        __syncthreads();
    }
    mx = max(mx, __shfl_xor(mx, 32));

    RowIndex<MODE> ri; // exact index map for this lane's row, applied to raw scores
    ri.init(hp, mx, top);

    // ================================================================= sweep B: row sum of E_hat
    const uint8_t *lut_b = lut_lds;
    uint32_t sum = 0;
    v16i cs = zero16; // V column sums of channel block `wave` (needed by sweep C's signed bytes)
    const v4i ones = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};

    // element-wise stage of sweep B on one finished score block
    auto valu_b = [&](auto masked_tag, const v16i &s, int klo) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (MASKED) {
                const uint32_t e = lut_b[ri(min(max(s[i], ri.bound), ri.mx))]; // hidden keys may exceed the max
                sum += visible(klo + acc_key(i, h)) ? e : 0u;
            } else {
                sum += lut_b[ri(max(s[i], ri.bound))];
            }
        }
    };

    auto stage_next = [&](int t) { // end of iteration t: publish tile t+1, start fetching tile t+2
        if (t + 1 < ntiles) {
            store_k(t + 1);
            store_v(t + 1);
        }
        if (t + 2 < ntiles) {
            load_k(t + 2);
            load_v(t + 2);
        }
        __syncthreads();
    };
    auto sweep_prologue = [&]() {
        load_k(0);
        load_v(0);
        store_k(0);
        store_v(0);
        if (ntiles > 1) {
            load_k(1);
            load_v(1);
        }
        __syncthreads();
    };
    auto colsum_step = [&](int t) {
        if (wave < CB) {
            cs = __builtin_amdgcn_mfma_i32_32x32x32_i8(vt_frag(Vs[t % NBUF], 0, wave), ones, cs, 0, 0, 0);
            cs = __builtin_amdgcn_mfma_i32_32x32x32_i8(vt_frag(Vs[t % NBUF], 1, wave), ones, cs, 0, 0, 0);
        }
    };

    if (INTATTN_PROFILE_SWEEPS & 2) {
        sweep_prologue();
        // hot loop: tiles wholly visible to this wave, no masks, software-pipelined
        v16i sA = qk(Ks[0], 0, zero16), sB;
        for (int t = 0; t < nfull; ++t) {
            const int8_t *kcur = Ks[t % NBUF], *knext = Ks[(t + 1) % NBUF];
            // step 0: score block (t, 1) on the matrix core while block (t, 0) goes through the ALU
            sB = qk(kcur, 1, zero16);
            valu_b(std::false_type{}, sA, 0);
            colsum_step(t);
            stage_next(t);
            // step 1: block (t+1, 0) on the matrix core (recomputed by the tail loop if masked)
            sA = qk(knext, 0, zero16);
            valu_b(std::false_type{}, sB, 0);
        }
        // tail: the diagonal / ragged / hidden tiles of this wave, masked, not pipelined
        for (int t = nfull; t < ntiles; ++t) {
            const int8_t *kcur = Ks[t % NBUF];
            if (!(CAUSAL && t * BK > qw0 + 31)) {
                const v16i s0 = qk(kcur, 0, zero16), s1 = qk(kcur, 1, zero16);
                valu_b(std::true_type{}, s0, t * BK);
                valu_b(std::true_type{}, s1, t * BK + 32);
            }
            colsum_step(t);
            stage_next(t);
        }
    }
    if (wave < CB && n == 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) colsum[32 * wave + acc_key(i, h)] = cs[i];
    }
    sum += __shfl_xor(sum, 32);
    if (sum == 0) sum = 1; // only rows beyond L; never stored
    {
        // per-row probability table: PT[idx] = round(255 * LUT_hat[idx] / sum) - 128 as a byte
        uint32_t *pt = PT[wave];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int kidx = 16 * h + j;
            const uint32_t e = lut_b[kidx];
            const uint32_t pr = (510u * e + sum) / (2u * sum);
            pt[kidx * 32 + n] = (pr ^ 0x80u) & 0xffu;
        }
        if (p.dbg_row_max && h == 0 && row < L) p.dbg_row_max[(int64_t)bh * L + row] = mx;
        if (p.dbg_row_sum && h == 0 && row < L) p.dbg_row_sum[(int64_t)bh * L + row] = (int32_t)sum;
    }

    // ================================================================= sweep C: P_hat and P_hat.V_hat
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) o[cb] = zero16;

    const uint32_t *pt = PT[wave] + n;
    // element-wise stage of sweep C: 16 probability bytes (minus 128) = one MFMA B operand
    auto valu_c = [&](auto masked_tag, const v16i &s, int klo) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        v4i pf;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t pb4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 4 * g + r;
                if (MASKED) {
                    const uint32_t pb = pt[ri(min(max(s[i], ri.bound), ri.mx)) * 32];
                    pb4[r] = visible(klo + acc_key(i, h)) ? pb : 0x80u;
                } else {
                    pb4[r] = pt[ri(max(s[i], ri.bound)) * 32];
                }
            }
            pf[g] = (int)(((pb4[1] << 8) | pb4[0]) | (((pb4[3] << 8) | pb4[2]) << 16));
        }
        return pf;
    };
    auto pv = [&](const int8_t *vbuf, int st, const v4i &pf) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
            o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vt_frag(vbuf, st, cb), pf, o[cb], 0, 0, 0);
    };

    if (INTATTN_PROFILE_SWEEPS & 4) {
        sweep_prologue();
        v16i sA = qk(Ks[0], 0, zero16), sB;
        v4i pfA, pfB = v4i{0, 0, 0, 0}; // zero bytes: the first, dangling P.V step adds nothing
        for (int t = 0; t < nfull; ++t) {
            const int8_t *kcur = Ks[t % NBUF], *knext = Ks[(t + 1) % NBUF];
            const int8_t *vcur = Vs[t % NBUF], *vprev = Vs[(t + NBUF - 1) % NBUF];
            // step 0: matrix core: scores (t, 1) and P.V of block (t-1, 1); ALU: block (t, 0)
            sB = qk(kcur, 1, zero16);
            pv(vprev, 1, pfB);
            pfA = valu_c(std::false_type{}, sA, 0);
            stage_next(t);
            // step 1: matrix core: scores (t+1, 0) and P.V of block (t, 0); ALU: block (t, 1)
            sA = qk(knext, 0, zero16);
            pv(vcur, 0, pfA);
            pfB = valu_c(std::false_type{}, sB, 0);
        }
        if (nfull > 0) pv(Vs[(nfull - 1) % NBUF], 1, pfB);
        // tail: every wave walks every remaining tile (the column-sum correction assumes it)
        for (int t = nfull; t < ntiles; ++t) {
            const int8_t *kcur = Ks[t % NBUF], *vcur = Vs[t % NBUF];
            const v16i s0 = qk(kcur, 0, zero16), s1 = qk(kcur, 1, zero16);
            const v4i pf0 = valu_c(std::true_type{}, s0, t * BK);
            const v4i pf1 = valu_c(std::true_type{}, s1, t * BK + 32);
            pv(vcur, 0, pf0);
            pv(vcur, 1, pf1);
            stage_next(t);
        }
    }

    // ================================================================= epilogue
    // colsum was written after sweep B; sweep C's barriers made it visible
    if (row < L) {
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
}

template <int D, bool CAUSAL>
int launch_pipe_mode(const FwdParams &p, int idx_mode, hipStream_t st)
{
    const dim3 grid((unsigned)fwd_grid_size(p.B, p.Hq, p.Hkv, p.n_qtiles)), block(NT);
    if (idx_mode == IDX_MAD24)
        hipLaunchKernelGGL((fwd_pipe_kernel<D, CAUSAL, IDX_MAD24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_MULHI24)
        hipLaunchKernelGGL((fwd_pipe_kernel<D, CAUSAL, IDX_MULHI24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_FP32)
        hipLaunchKernelGGL((fwd_pipe_kernel<D, CAUSAL, IDX_FP32>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((fwd_pipe_kernel<D, CAUSAL, IDX_DIV>), grid, block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

int launch_fwd_pipe(const FwdParams &p, int d, int idx_mode, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (d == 64) return p.causal ? launch_pipe_mode<64, true>(p, idx_mode, st) : launch_pipe_mode<64, false>(p, idx_mode, st);
    if (d == 128) return p.causal ? launch_pipe_mode<128, true>(p, idx_mode, st) : launch_pipe_mode<128, false>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
