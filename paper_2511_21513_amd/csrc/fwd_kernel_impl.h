// Fused IntAttention forward for gfx950 (MI355X).
//
// One workgroup = 4 wavefronts; each wavefront owns RB blocks of 32 query rows of one
// (batch, query head).  Keys/values stream through LDS in tiles of BK keys, double
// buffered, one barrier per tile.  Because IndexSoftmax (Sec. 3.1-3.2) needs the exact row
// maximum before any table index and the exact row sum before any probability, the key axis
// is swept three times, recomputing the INT8 score tile each time instead of ever storing
// the L x L matrix:
//   sweep A: S^T = K.Q^T (MFMA)            -> running row max
//   sweep B: S^T again -> clip, index (the row max is folded into per-row constants), LUT_hat ->
//            row sum; then the 2^b distinct probabilities of the row, P_hat = round(255 E/S), go
//            to a per-row table in LDS
//   sweep C: S^T again -> index -> per-row table -> 16 probability bytes per lane, which
//            are exactly one MFMA B operand of O^T += V^T.P^T; then requantize and store.
// Scores are produced transposed (keys x queries) so that each lane owns one query row:
// row max and row sum are in-lane plus one exchange between the two half-waves.
//
// The int8 MFMA is signed x signed while P_hat is unsigned (0..255).  The kernel feeds
// P_hat - 128 and adds 128 * (column sums of the V rows of every processed tile) at the end;
// hidden keys inside a processed tile carry P_hat = 0, i.e. the byte -128, so the correction
// is the plain column sum.  colsum_kernel (below) leaves the sums of V over each chunk of as
// many keys as a workgroup has query rows; sweep C adds up the chunks it covers.  All
// intermediate magnitudes stay below 2^31 for L < 131072.
//
// LDS tiles are row-major [key][d] with the 16-byte chunks of each row XOR-swizzled so that
// both access patterns are bank-conflict free: K fragments are read with 128-bit loads
// (one key row per lane), V^T fragments with the transposing 64-bit load (eight key rows per
// 16 lanes).  The tiles are filled by buffer loads that write LDS directly.
//
// Within a tile the work is ordered in phases (all fragment reads, all MFMAs, all index
// arithmetic with every table lookup in flight, then the consumers).  This is the kernel for
// small problems (all three sweeps in one launch) and for sweeps A+B of large ones; sweep C of
// large problems has a software-pipelined kernel of its own.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace fwdk {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;

// PH selects which part of the path this instantiation runs: 0 = all three sweeps in one launch;
// 1 = sweeps A and B only (row max and row sum go to a small workspace: 8 bytes per query row) --
// without the output accumulators it needs far fewer registers, so a wave can own 64 query rows
// (every K fragment read feeds two MFMAs) at three waves per SIMD; 2 = sweep C only, reading that
// workspace.
template <int D, int RB, int KT, bool CAUSAL, int MODE, int PH>
__global__ __launch_bounds__(NT, PH == 1 ? (RB * KT <= 2 ? 4 : 3) : (RB == 1 ? (KT == 1 ? 3 : 2) : 1)) void fwd_kernel(const FwdParams p)
{
    constexpr int KS = KT; // sub-tiles sweep C computes per step: the whole staged tile
    constexpr int KB = D / 32;       // 32-wide blocks of the head dimension
    constexpr int CB = D / 32;       // 32-wide blocks of output channels
    constexpr int BK = 32 * KT;      // keys per tile
    constexpr int BQ = WAVES * RB * 32;
    constexpr int TILE = BK * D;     // bytes
    constexpr int NBLK = TILE / 1024;                // 1 KiB blocks per tile (one wave-wide 16-byte load each)
    constexpr int JB = (NBLK + WAVES - 1) / WAVES;   // blocks per wave per tile
    constexpr int CPR = D / 16;                      // 16-byte chunks per key row
    constexpr int RPB = 1024 / D;                    // key rows per block

    // Two buffers per operand, as separate arrays: the compiler tracks each direct-to-LDS load by
    // the array it targets, so reads of one buffer need not wait for loads into the other.
    __shared__ __attribute__((aligned(1024))) int8_t Ks0[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Ks1[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Vs0[PH == 1 ? 16 : TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Vs1[PH == 1 ? 16 : TILE];
    // per-row probability tables, [wave][row block][idx][row]: dynamic shared memory of WAVES * RB * NIDX * 32
    // words, NIDX = 32 or 64 table entries (none for sweeps A+B alone)
    extern __shared__ uint32_t PT[];
    __shared__ uint32_t lut_lds[16];
    __shared__ int32_t colsum[D];
    __shared__ int32_t cs4[PH == 0 ? WAVES : 1][D]; // in-kernel column sums of V (short sequences, single launch)

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return; // padding of the XCD-aware grid (uniform for the whole workgroup)
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt + p.row_lo / BQ;
    const int bh = b * p.Hq + hq;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    // device-derived parameters: another launch of this pair serves the head when its scheme is not this
    // kernel's (uniform for the workgroup); the top-byte scheme runs in the multiply-add code here
    if (p.filter && (hp.pad[0] == IDX_TOP24 ? (int)IDX_MAD24 : hp.pad[0]) != MODE) return;
    const int L = p.Lk; // keys
    // query rows: [rlo, rhi) of the numbering in which row r sees keys <= r under the causal mask
    const int rlo = p.row_lo, rhi = p.row_lo + p.L, LQ = p.L;
    const uint32_t top = (uint32_t)p.top;
    const int NIDX = top < 32 ? 32 : 64; // table entries allocated per row
    // Finer quantization groups over both axes (Sec. 3.3): the lane's query row has the scale of its block
    // of q_block rows, every key the scale of its block of k_block keys.  alpha^(g) = s_Q^(g) s_K^(g) / sqrt(d)
    // per logit; the row maximum is taken over the dequantized logits (fp64), and each key block measures
    // distances from the image of that maximum in its own integer units.
    constexpr bool KG = MODE == IDX_KGROUP;
    const float *skp = KG ? p.sk_blocks + (int64_t)(b * p.Hkv + kvh) * p.n_kblk : nullptr;
    const bool kg_blocks = KG && (p.k_block % 32) == 0; // a 32-key sub-tile lies in one key block (uniform)
    double sq_row[RB], Mreal[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        sq_row[rb] = 0.0;
        Mreal[rb] = -__builtin_inf();
    }

    const int q0 = qt * BQ, qw0 = q0 + wave * (RB * 32);
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    if (tid < 16) lut_lds[tid] = p.lut[tid];
    if constexpr (KG) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = q0 + wave * (RB * 32) + 32 * rb + n;
            const int lr = (row >= rlo && row < rhi) ? row - rlo : 0;
            sq_row[rb] = (double)p.sq_rows[(int64_t)bh * p.n_rowblk + lr / p.q_block];
        }
    }
    // alpha^(g) of the logit (lane's row of row block rb, key); keys past the end take the last block's scale
    auto kg_alpha = [&](int rb, int key) __attribute__((always_inline)) {
        return (sq_row[rb] * (double)skp[min(key, L - 1) / p.k_block]) / p.sqrt_d;
    };

    // Q fragments: row block rb, row qw0 + 32 rb + n, bytes [32 kb + 16 h, +16).
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

    // ---- staging: global -> LDS directly (no registers, no LDS store instructions), a tile ahead.
    // One wave-wide 16-byte load fills 1 KiB of LDS, lane i at byte 16 i: the lane's slot is key row
    // i / CPR of the block at chunk position i % CPR, which under the XOR swizzle holds global chunk
    // (i % CPR) ^ swz(key) -- so the swizzle is applied to the global address.
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
    // One sweep over the key tiles: tile t+1 is requested before tile t is computed; the barrier at
    // the end of a step (which waits for the wave's own loads first) publishes it and frees tile
    // t's buffer.  Unrolled by two so that every buffer is named statically.
    auto sweep = [&](auto with_v, auto body) __attribute__((always_inline)) {
        constexpr bool WITH_V = decltype(with_v)::value;
        dma_k(0, Ks0);
        if (WITH_V) dma_v(0, Vs0);
        publish_tiles_barrier();
        for (int t = 0; t < ntiles; t += 2) {
            if (t + 1 < ntiles) {
                dma_k(t + 1, Ks1);
                if (WITH_V) dma_v(t + 1, Vs1);
            }
            body(t, (const int8_t *)Ks0, (const int8_t *)Vs0);
            publish_tiles_barrier();
            if (t + 1 < ntiles) {
                if (t + 2 < ntiles) {
                    dma_k(t + 2, Ks0);
                    if (WITH_V) dma_v(t + 2, Vs0);
                }
                body(t + 1, (const int8_t *)Ks1, (const int8_t *)Vs1);
                publish_tiles_barrier();
            }
        }
    };

    // ---- S^T blocks of one tile: KT sub-tiles of 32 keys x RB row blocks, KB chained MFMAs each.
    // The chains are interleaved (kb outermost) so that consecutive MFMAs are independent.
    // All K fragments of the tile are requested before the first MFMA (the scheduling barrier keeps
    // the compiler from re-serialising read -> wait -> MFMA), so one LDS latency is paid per tile.
    auto qk_tile = [&](const int8_t *Kb, int st0, auto &s) __attribute__((always_inline)) {
        constexpr int NS = (int)(sizeof(s) / sizeof(s[0]));
        v4i kf[KB][NS];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                const int key = 32 * (st0 + st) + n;
                kf[kb][st] = *(const v4i *)(Kb + key * D + (((2 * kb + h) ^ swz_k<D>(key)) << 4));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int st = 0; st < NS; ++st) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    s[st][rb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb][st], qf[rb][kb], s[st][rb], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto visible = [&](int key, int row) { return key < L && (!CAUSAL || key <= row); };
    // wave-uniform: every key of tile t is visible to every row of this wave (no mask needed)
    auto tile_is_full = [&](int t) { return (t + 1) * BK <= L && (!CAUSAL || (t + 1) * BK - 1 <= qw0); };
    // wave-uniform: no key of tile t is visible to any row of this wave
    auto tile_is_hidden = [&](int t) { return CAUSAL && t * BK > qw0 + RB * 32 - 1; };

    // ================================================================= sweep A: row max
    int mx[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) mx[rb] = INT32_MIN;

    auto tile_a = [&](auto masked_tag, int t, const int8_t *Kb) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        v16i s[KT][RB];
#pragma unroll
        for (int st = 0; st < KT; ++st)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[st][rb][i] = 0;
        qk_tile(Kb, 0, s);
#pragma unroll
        for (int st = 0; st < KT; ++st) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if constexpr (KG) {
                    const int klo = t * BK + 32 * st, row = qw0 + 32 * rb + n;
                    if (kg_blocks) {
                        int lmax = INT32_MIN; // no score is INT32_MIN
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            if (!MASKED || visible(klo + acc_key(i, h), row)) lmax = max(lmax, s[st][rb][i]);
                        if (lmax != INT32_MIN) {
                            const double x = kg_alpha(rb, klo) * (double)lmax; // alpha > 0: the block's largest logit
                            Mreal[rb] = x > Mreal[rb] ? x : Mreal[rb];
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int key = klo + acc_key(i, h);
                            if (!MASKED || visible(key, row)) {
                                const double x = kg_alpha(rb, key) * (double)s[st][rb][i];
                                Mreal[rb] = x > Mreal[rb] ? x : Mreal[rb];
                            }
                        }
                    }
                } else if (MASKED) {
                    const int klo = t * BK + 32 * st, row = qw0 + 32 * rb + n;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        mx[rb] = visible(klo + acc_key(i, h), row) ? max(mx[rb], s[st][rb][i]) : mx[rb];
                } else {
#pragma unroll
                    for (int i = 0; i < 16; i += 2) mx[rb] = max(max(s[st][rb][i], s[st][rb][i + 1]), mx[rb]);
                }
            }
        }
    };

    if constexpr (PH != 2) {
        sweep(std::false_type{}, [&](int t, const int8_t *Kb, const int8_t *) __attribute__((always_inline)) {
            if (tile_is_full(t)) tile_a(std::false_type{}, t, Kb);
            else if (!tile_is_hidden(t)) tile_a(std::true_type{}, t, Kb);
        });
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) mx[rb] = max(mx[rb], __shfl_xor(mx[rb], 32));
        if constexpr (KG) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const double o = __shfl_xor(Mreal[rb], 32);
                Mreal[rb] = o > Mreal[rb] ? o : Mreal[rb];
            }
        }
    } else {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = qw0 + 32 * rb + n;
            mx[rb] = (row >= rlo && row < rhi) ? p.ws_row_max[(int64_t)bh * LQ + (row - rlo)] : 0;
        }
    }

    // exact index map of each row block's lane row, applied to raw scores (no -rowMax start
    // value in the accumulators, which saves 16 registers per row block)
    // parameters of the block of query rows that `row` lies in (finer groups over query rows, Sec. 3.3)
    auto row_hp = [&](int row) __attribute__((always_inline)) {
        const int lr = (row >= rlo && row < rhi) ? row - rlo : 0;
        return p.row_table[(int64_t)bh * p.n_rowblk + lr / p.q_block];
    };
    RowIndex<MODE> ri[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) ri[rb].init(MODE == IDX_ROW64 ? row_hp(qw0 + 32 * rb + n) : hp, KG ? 0 : mx[rb], top);
    if constexpr (KG) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) ri[rb].shift = (int)top; // bound of the index (see RowIndex)
    }
    // Key groups: the index constants of the lane's row for the key block of `key` (Sec. 3.3):
    // c_int^(g) = round(c / alpha^(g)) capped at 2^30, m^(g) = round(M / alpha^(g)), the fp64 index map's
    // factor for c_int^(g).  m^(g) is clamped to [-2^22, 2^30 + 2^22]: below every logit / far enough above
    // every logit that the distance exceeds any c_int, so the clamp changes no result and all later
    // arithmetic fits 32 bits (comparisons written so that a NaN from an unusable scale lands on a bound).
    auto kg_index = [&](int rb, int key) __attribute__((always_inline)) {
        const double al = kg_alpha(rb, key);
        double cd = __builtin_floor(p.clip / al + 0.5);
        cd = cd >= 1.0 ? cd : 1.0;
        cd = cd < 1073741824.0 ? cd : 1073741824.0;
        double md = __builtin_floor(Mreal[rb] / al + 0.5);
        md = md < 1077936128.0 ? md : 1077936128.0;
        md = md > -4194304.0 ? md : -4194304.0;
        const int c_int = (int)cd;
        ri[rb].mx = (int)md;
        ri[rb].bound = ri[rb].mx - c_int;
        const uint64_t bits = (uint64_t)__double_as_longlong((double)top / cd) + 1ull; // the double after top / c_int
        ri[rb].negr = __longlong_as_double((long long)(bits ^ 0x8000000000000000ull));
    };

    // ================================================================= sweep B: row sum of E_hat
    // transposing read: lanes 2j, 2j+1 of a 16-lane group point at the two 8-byte halves of key
    // row j's 16 channels; lane i of the group receives channel i of the eight rows.
    const int tr_i = lane & 15, tr_g = (lane >> 4) & 1;
    auto vt_frag = [&](const int8_t *Vb, int st, int cb) __attribute__((always_inline)) {
        v4i a;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int j = tr_i >> 1;
            const int key = 32 * st + 8 * (2 * r + (j >> 2)) + 4 * h + (j & 3);
            const int c16 = 2 * cb + tr_g;
            const int8_t *ptr = Vb + key * D + ((c16 ^ swz_v<D>(key)) << 4) + 8 * (tr_i & 1);
            const v2i x = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)ptr);
            a[2 * r] = x[0];
            a[2 * r + 1] = x[1];
        }
        return a;
    };

    const uint8_t *lut_b = (const uint8_t *)lut_lds;
    uint32_t sum[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) sum[rb] = 0;

    auto tile_b = [&](auto masked_tag, int t, const int8_t *Kb) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        v16i s[KT][RB];
#pragma unroll
        for (int st = 0; st < KT; ++st)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[st][rb][i] = 0;
        qk_tile(Kb, 0, s);
#pragma unroll
        for (int st = 0; st < KT; ++st) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if constexpr (KG) {
                    const int klo = t * BK + 32 * st, row = qw0 + 32 * rb + n;
                    if (kg_blocks) kg_index(rb, klo);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int key = klo + acc_key(i, h);
                        if (!kg_blocks) kg_index(rb, key);
                        const uint32_t e = lut_b[ri[rb](min(max(s[st][rb][i], ri[rb].bound), ri[rb].mx))];
                        sum[rb] += (!MASKED || visible(key, row)) ? e : 0u;
                    }
                } else if (MASKED) {
                    const int klo = t * BK + 32 * st, row = qw0 + 32 * rb + n;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        // hidden keys may exceed the row max
                        const uint32_t e = lut_b[ri[rb](min(max(s[st][rb][i], ri[rb].bound), ri[rb].mx))];
                        sum[rb] += visible(klo + acc_key(i, h), row) ? e : 0u;
                    }
                } else {
                    // every lookup of the block is issued before the first one is consumed
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[st][rb][i] = (int)lut_b[ri[rb](max(s[st][rb][i], ri[rb].bound))];
                }
            }
        }
        if (!MASKED && !KG) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int st = 0; st < KT; ++st)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sum[rb] += (uint32_t)s[st][rb][i];
        }
    };

    if constexpr (PH != 2) {
        sweep(std::false_type{}, [&](int t, const int8_t *Kb, const int8_t *) __attribute__((always_inline)) {
            if (tile_is_full(t)) tile_b(std::false_type{}, t, Kb);
            else if (!tile_is_hidden(t)) tile_b(std::true_type{}, t, Kb);
        });
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) sum[rb] += __shfl_xor(sum[rb], 32);
    }
    if constexpr (PH == 1) {
        // hand row max and row sum to the second launch
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = qw0 + 32 * rb + n;
            if (h == 0 && row >= rlo && row < rhi) {
                p.ws_row_max[(int64_t)bh * LQ + (row - rlo)] = mx[rb];
                p.ws_row_sum[(int64_t)bh * LQ + (row - rlo)] = (int32_t)sum[rb];
            }
        }
        return;
    } else if constexpr (PH == 2) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = qw0 + 32 * rb + n;
            sum[rb] = (row >= rlo && row < rhi) ? (uint32_t)p.ws_row_sum[(int64_t)bh * LQ + (row - rlo)] : 0u;
        }
    }
    // Column sums of V over every key that sweep C's tiles cover (keys up to the end of this query
    // tile under the causal mask, else all): the correction for feeding the probabilities to the
    // signed MFMA as P - 128.  A small kernel ahead of this one left the sums of each BQ-key chunk
    // per (batch, KV head); visible to all waves after sweep C's barriers.
    if (PH != 0 || p.ws_colsum) {
        if (tid < D) {
            const int32_t *cp = p.ws_colsum + (int64_t)(b * p.Hkv + kvh) * p.n_chunks * D + tid;
            const int nchunk = CAUSAL ? min(qt + 1, p.n_chunks) : p.n_chunks;
            int32_t acc = 0;
#pragma unroll 8
            for (int c = 0; c < nchunk; ++c) acc += cp[(int64_t)c * D];
            colsum[tid] = acc;
        }
    } else {
        // Short key sequences: the launch of the small kernel costs more than summing V over the
        // keys [0, kmax) here (thread = 16 channels of every KL-th key row, then the key lanes of
        // a wave by lane exchange, then the four waves through LDS).
        constexpr int G = D / 16, KL = NT / G;
        const int c16 = tid % G, kl = tid / G;
        int32_t a16[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) a16[i] = 0;
        for (int key = kl; key < kmax; key += KL) {
            const v4i x = *(const v4i *)(Vp + (int64_t)key * p.vs[2] + c16 * 16);
#pragma unroll
            for (int i = 0; i < 16; ++i) a16[i] += (int32_t)(int8_t)((uint32_t)x[i / 4] >> (8 * (i % 4)));
        }
#pragma unroll
        for (int o = G; o < 64; o <<= 1)
#pragma unroll
            for (int i = 0; i < 16; ++i) a16[i] += __shfl_xor(a16[i], o);
        if (lane < G)
#pragma unroll
            for (int i = 0; i < 16; ++i) cs4[wave][c16 * 16 + i] = a16[i];
        __syncthreads();
        if (tid < D) colsum[tid] = cs4[0][tid] + cs4[1][tid] + cs4[2][tid] + cs4[3][tid];
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (sum[rb] == 0) sum[rb] = 1; // only rows outside [rlo, rhi); never stored
        // per-row probability table: PT[idx] = round(255 * LUT_hat[idx] / sum) - 128 as a byte
        uint32_t *pt = PT + (wave * RB + rb) * NIDX * 32;
        const float inv_2s = __builtin_amdgcn_rcpf((float)(2u * sum[rb]));
        for (int j = 0; j < NIDX / 2; ++j) {
            const int kidx = (NIDX / 2) * h + j;
            pt[kidx * 32 + n] = (prob_u8(lut_b[kidx], sum[rb], inv_2s) ^ 0x80u) & 0xffu;
        }
        const int row = qw0 + 32 * rb + n;
        if (!KG && p.dbg_row_max && h == 0 && row >= rlo && row < rhi) p.dbg_row_max[(int64_t)bh * LQ + (row - rlo)] = mx[rb];
        if (p.dbg_row_sum && h == 0 && row >= rlo && row < rhi) p.dbg_row_sum[(int64_t)bh * LQ + (row - rlo)] = (int32_t)sum[rb];
    }

    // ================================================================= sweep C: P_hat and P_hat.V_hat
    v16i o[RB][CB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[rb][cb][i] = 0;

    // One tile of sweep C in phases, separated by scheduling barriers so that each kind of LDS
    // latency is paid once per tile: S^T blocks; all probability lookups (in place, one per score)
    // followed by all V^T fragment reads; packing into MFMA B operands (LDS returns in order, so
    // the lookups land first while the fragments are still in flight).
    auto tile_c = [&](auto masked_tag, int t, const int8_t *Kb, const int8_t *Vb, int st0, v4i (&pf)[KS][RB],
                      v4i (&vf)[KS][CB]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        v16i s[KS][RB];
#pragma unroll
        for (int st = 0; st < KS; ++st)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[st][rb][i] = 0;
        qk_tile(Kb, st0, s);
#pragma unroll
        for (int st = 0; st < KS; ++st) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const uint32_t *pt = PT + (wave * RB + rb) * NIDX * 32 + n;
                if (kg_blocks) kg_index(rb, t * BK + 32 * (st0 + st));
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (KG && !kg_blocks) kg_index(rb, t * BK + 32 * (st0 + st) + acc_key(i, h));
                    const int sc = (MASKED || KG) ? min(max(s[st][rb][i], ri[rb].bound), ri[rb].mx) : max(s[st][rb][i], ri[rb].bound);
                    s[st][rb][i] = (int)pt[ri[rb](sc) * 32];
                }
            }
        }
#pragma unroll
        for (int st = 0; st < KS; ++st)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) vf[st][cb] = vt_frag(Vb, st0 + st, cb);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < KS; ++st) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const int klo = t * BK + 32 * (st0 + st), row = qw0 + 32 * rb + n;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t pb4[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 4 * g + r;
                        pb4[r] = (uint32_t)s[st][rb][i];
                        if (MASKED) pb4[r] = visible(klo + acc_key(i, h), row) ? pb4[r] : 0x80u;
                    }
                    pf[st][rb][g] = (int)(((pb4[1] << 8) | pb4[0]) | (((pb4[3] << 8) | pb4[2]) << 16));
                }
            }
        }
    };

    // every wave walks every tile of the workgroup here: the column-sum correction assumes it
    sweep(std::true_type{}, [&](int t, const int8_t *Kb, const int8_t *Vb) __attribute__((always_inline)) {
#pragma unroll
        for (int st0 = 0; st0 < KT; st0 += KS) {
            // (the P_hat.V_hat MFMAs follow in one place for both instantiations, so that the output
            // accumulators have a single home)
            v4i pf[KS][RB], vf[KS][CB];
            // wave-uniform: every key of this step is visible to every row of this wave
            const int khi = t * BK + 32 * (st0 + KS);
            if (khi <= L && (!CAUSAL || khi - 1 <= qw0)) tile_c(std::false_type{}, t, Kb, Vb, st0, pf, vf);
            else tile_c(std::true_type{}, t, Kb, Vb, st0, pf, vf);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int st = 0; st < KS; ++st) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        o[rb][cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[st][cb], pf[st][rb], o[rb][cb], 0, 0, 0);
                }
            }
        }
    });

    // ================================================================= epilogue
    // colsum was written after sweep B; sweep C's barriers made it visible
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = qw0 + 32 * rb + n;
        if (row < rlo || row >= rhi) continue;
        int8_t *Op = p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)(row - rlo) * p.os[2];
        HeadParams he = (MODE == IDX_ROW64 || KG) ? row_hp(row) : hp;
        if (KG && p.head_status[hq] != 0) he.rq_mult = 0; // an unusable scale somewhere in the head: all zeros
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch0 = cb * 32 + 8 * g + 4 * h;
                uint32_t packed = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int32_t acc = o[rb][cb][4 * g + r] + 128 * colsum[ch0 + r];
                    if (p.dbg_acc) p.dbg_acc[((int64_t)bh * LQ + (row - rlo)) * D + ch0 + r] = acc;
                    packed |= ((uint32_t)requant_any(acc, he.rq_mult, he.rq_shift) & 0xffu) << (8 * r);
                }
                *(uint32_t *)(Op + ch0) = packed;
            }
        }
    }
}

template <int D, int RB, int KT, bool CAUSAL, int PH>
int launch_mode(const FwdParams &p, int idx_mode, hipStream_t st)
{
    const dim3 grid((unsigned)fwd_grid_size(p.B, p.Hq, p.Hkv, p.n_qtiles)), block(NT);
    // dynamic shared memory: the per-row probability tables (32 or 64 entries of a word per query row)
    const unsigned sh = PH == 1 ? 0u : (unsigned)(WAVES * RB * (p.top < 32 ? 32 : 64) * 32 * sizeof(uint32_t));
    if (idx_mode == IDX_DEVICE) {
        // the scheme of each head is known on the device only: one launch per scheme, each
        // skipping the heads of the other
        FwdParams pf = p;
        pf.filter = 1;
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_MAD24, PH>), grid, block, sh, st, pf);
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_FP64, PH>), grid, block, sh, st, pf);
        return (int)hipGetLastError();
    }
    if constexpr (RB == 1 && KT == 2 && PH == 0) {
        if (idx_mode == IDX_KGROUP) { // groups over the key axis: single-launch kernel only
            hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_KGROUP, PH>), grid, block, sh, st, p);
            return (int)hipGetLastError();
        }
    }
    if (idx_mode == IDX_KGROUP) return (int)hipErrorInvalidValue;
    if (idx_mode == IDX_MAD24 || idx_mode == IDX_TOP24) // TOP24 is MAD24 with the shift at 24: same code here
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_MAD24, PH>), grid, block, sh, st, p);
    else if (idx_mode == IDX_MULHI24)
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_MULHI24, PH>), grid, block, sh, st, p);
    else if (idx_mode == IDX_FP32)
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_FP32, PH>), grid, block, sh, st, p);
    else if (idx_mode == IDX_ROW64)
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_ROW64, PH>), grid, block, sh, st, p);
    else
        hipLaunchKernelGGL((fwd_kernel<D, RB, KT, CAUSAL, IDX_FP64, PH>), grid, block, sh, st, p);
    return (int)hipGetLastError();
}

template <int RB, int KT, int PH>
int launch_shape(const FwdParams &p, int d, int idx_mode, hipStream_t st)
{
    if (d == 64)
        return p.causal ? launch_mode<64, RB, KT, true, PH>(p, idx_mode, st) : launch_mode<64, RB, KT, false, PH>(p, idx_mode, st);
    if (d == 128)
        return p.causal ? launch_mode<128, RB, KT, true, PH>(p, idx_mode, st) : launch_mode<128, RB, KT, false, PH>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace fwdk

} // namespace intattn
