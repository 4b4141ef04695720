// Sweep C of the IntAttention forward as a kernel of its own (gfx950): with the row maxima and row
// sums of E_hat already in a workspace, recompute the INT8 scores, map them through the index
// map and the per-row probability table (Sec. 3.1-3.2: P_hat = round(255 E_hat / S)), multiply
// by V_hat on the matrix cores and requantize (INT8 output).
//
// Same data layout and lane ownership as the generic forward kernel (transposed scores, one query
// row per lane, XOR-swizzled K/V tiles in LDS filled by direct global->LDS loads); a wave owns RB
// blocks of 32 query rows.  What differs is the instruction schedule.  The generic kernel runs a
// tile as phases (scores, lookups, pack, P.V), so the matrix core idles during the vector phases
// and the other way round.  Here the key axis is walked in steps of 32 keys as a software
// pipeline inside each wave, meant to keep one wave per SIMD busy on its own (512 registers, the
// output accumulators in the accumulator half).  Step j issues
//     one MFMA, then the vector work of EPS scores, one MFMA, ...:
//   MFMAs:   the scores of sub-tile j+1 (KB chained MFMAs per row block), then P.V of sub-tile j-1
//   vector:  clip/index/table lookup (issued, not awaited) of sub-tile j's scores, and the packing
//            into MFMA operands of the probability bytes looked up half a step earlier
//   LDS:     K fragments of sub-tile j+2 (once the current ones are consumed), V^T fragments of
//            sub-tile j (after the last P.V of j-1 has issued)
// so every MFMA runs under independent vector instructions of the same wave, every LDS result
// has half a step or more to arrive, and nothing waits on what it has just issued.  Scheduling
// barriers pin that order.
//
// Table lookups without LDS.  P_hat = round(255 E_hat / S) is 0 for every table index k with
// 510 LUT_hat[k] < S (Eq. uint8-prob), so a row whose sum S exceeds 510 LUT_hat[8 n] can only give a
// nonzero probability at its first 8 n table entries, and once S > 510 every probability fits a
// signed byte.  Such a row keeps those entries in 2 n registers (n = 1, 2, 3), the kernel clips the
// distance at the first value whose index is 8 n instead of at c_int (the index map below that is
// unchanged), packs four index bytes into a register and looks four probabilities up with n byte
// permutes: a permute selects among the 8 bytes of a register pair, returns 0xff for selectors from 13
// up and 0 for selector 12 or a sign selector of a byte below 128, so with selectors rewritten per
// pair (in range: 0..7; out of range: >= 16) the AND of the n results is the entry, and the clipped
// index lands on a selector that yields 0.  No table in LDS, no lookup latency to hide, no offset of
// 128, no column-sum correction.  The LDS pipe is shared by the four SIMDs of a compute unit and a
// wave-wide byte lookup costs it three cycles -- sixteen of them per 32 x 32 block were the largest
// single cost of this kernel.  The path is chosen per wave: the largest n among its 32 rows, and the
// general path with the tables in LDS when a row has S <= 510 or more than 24 live entries.  The four
// waves of a workgroup meet at a barrier per tile, so a workgroup runs at the pace of its slowest wave:
// rows with similar sums (flat logits, encoder-style attention over many keys) gain up to a quarter,
// workloads whose row sums vary widely inside every tile (heavy-tailed logits) stay at the general
// path's speed.  (Sorting the rows of a tile by n to make its waves homogeneous was measured and
// dropped: the slowest wave still sets the pace.)
//
// Tiles are NSUB sub-tiles (64 or 128 keys), double buffered per operand; one barrier per tile.
// The K fragments are read two sub-tiles ahead of the V^T fragments.  K tiles are cut NSUB - 2
// sub-tiles earlier than V tiles (K tile t covers sub-tiles [NSUB (t-1) + 2, NSUB t + 2)), so that
// iteration T reads exactly K tile T+1 and V tile T, and at its top requests K tile T+2 and V
// tile T+1 into the buffers that were read an iteration ago.
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
__global__ __launch_bounds__(NT, RB == 1 ? 2 : 1) void sweep_c_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;       // 32-wide blocks of the head dimension
    constexpr int CB = D / 32;       // 32-wide blocks of output channels
    constexpr int NSUB = 4;          // sub-tiles (pipeline steps) per tile: long enough to cover the latency of the loads
    constexpr int KSHIFT = NSUB - 2; // K tiles start this many sub-tiles before V tiles (see above)
    constexpr int BK = 32 * NSUB;    // keys per tile
    constexpr int BQ = WAVES * RB * 32;
    constexpr int TILE = BK * D;     // bytes
    constexpr int SUB = 32 * D;      // bytes of a 32-key sub-tile
    constexpr int NBLK = TILE / 1024;
    constexpr int JB = (NBLK + WAVES - 1) / WAVES;
    constexpr int CPR = D / 16;
    constexpr int RPB = 1024 / D;
    constexpr int NSLOT = RB * (KB + CB); // MFMAs per step
    constexpr int NEL = 16 * RB;          // scores per lane and step
    constexpr int EPS = NEL / NSLOT;      // scores handled after each MFMA
    constexpr int HALF = NSLOT / 2;       // = RB * KB: P.V of sub-tile j-1 starts when its operands are complete
    static_assert(EPS == 2 || EPS == 4, "a slot handles half an operand register or a whole one");

    __shared__ __attribute__((aligned(1024))) int8_t Ks0[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Ks1[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Vs0[TILE];
    __shared__ __attribute__((aligned(1024))) int8_t Vs1[TILE];
    // per-row probability tables of the workgroup as bytes [idx][lane][wave]: a table row (one index) is 256
    // bytes, lane l of wave w owns byte 4 l + w of every row -- its own bank, so lookups never conflict --
    // and the address of an entry is (idx << 8) + 4 l + w, which the IDX_TOP24 scheme forms with one byte
    // permute.  The two lanes that share a query row (l and l + 32) each hold a copy of its table.
    static_assert(RB == 1 && WAVES == 4, "table layout: 64 lanes x 4 waves = one 256-byte row per index");
    // (aligned to 64 KiB: the table's address then has a zero byte 1 for the index to go into)
    __shared__ __attribute__((aligned(65536))) uint8_t PT[32 * 256];
    __shared__ uint32_t lut_lds[8];
    __shared__ int32_t colsum[D];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return; // padding of the XCD-aware grid (uniform for the whole workgroup)
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt + p.row_lo / BQ;
    const int bh = b * p.Hq + hq;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    if (MODE != IDX_MIX && p.filter && hp.pad[0] != MODE) return; // another launch of this pair serves the head (uniform for the workgroup)
    // The rest of the kernel with the index scheme M as a compile-time constant: MODE itself, or, under IDX_MIX,
    // the scheme named in the head's own parameters (top-byte constants where the head has them, else the
    // multiply-high scheme that serves every head of the call).
    auto body = [&](auto mode_tag) __attribute__((always_inline)) {
    constexpr int M = decltype(mode_tag)::value;
    const int L = p.Lk; // keys
    // query rows: [rlo, rhi) of the numbering in which row r sees keys <= r under the causal mask
    const int rlo = p.row_lo, rhi = p.row_lo + p.L, LQ = p.L;
    // parameters of the block of query rows that `row` lies in (finer groups over query rows, Sec. 3.3)
    auto row_hp = [&](int row) __attribute__((always_inline)) {
        const int lr = (row >= rlo && row < rhi) ? row - rlo : 0;
        return p.row_table[(int64_t)bh * p.n_rowblk + lr / p.q_block];
    };
    const uint32_t top = (uint32_t)p.top;

    const int q0 = qt * BQ;
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    if (tid < 8) lut_lds[tid] = p.lut[tid];

    const int kmax = CAUSAL ? min(L, q0 + BQ) : L;
    const int ntiles = (kmax + BK - 1) / BK; // iterations = V tiles; K tiles 0..ntiles are touched

    // ---- staging: direct global -> LDS loads; the XOR swizzle is applied to the global address
    // (lane i of a wave-wide 16-byte load lands at byte 16 i of its 1 KiB block).
    int dma_goff_k[JB], dma_goff_v[JB];
#pragma unroll
    for (int j = 0; j < JB; ++j) {
        const int key = (wave + WAVES * j) * RPB + lane / CPR, cp = lane % CPR;
        dma_goff_k[j] = key * (int)p.ks[2] + ((cp ^ swz_k<D>(key)) << 4); // the host checked BK * stride < 2^31
        dma_goff_v[j] = key * (int)p.vs[2] + ((cp ^ swz_v<D>(key)) << 4);
    }
    // The loads go through a buffer descriptor that starts at the tile's first key row and ends
    // with the last byte of key row L-1, so key rows at or past L come back as zeros from the range
    // check.  Blocks below first_blk are skipped (the part of K tile 0 that lies before key 0).
    auto dma_tile = [&](const int8_t *base, int64_t stride, const int (&goff)[JB], int key0, int first_blk, int8_t *dst)
                        __attribute__((always_inline)) {
        const int8_t *tb = base + (int64_t)key0 * stride; // wave-uniform
        const int64_t rem = (int64_t)(L - key0 - 1) * stride + D;
        const uint32_t nrec = rem <= 0 ? 0u : (rem > 0xffffffffll ? 0xffffffffu : (uint32_t)rem); // 0: all of it past L
#if defined(__HIP_DEVICE_COMPILE__) // the host pass has neither the descriptor type nor the builtins
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)tb, 0, (int)nrec, 0x00020000);
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int blk = wave + WAVES * j;
            if (blk < first_blk || (NBLK % WAVES != 0 && blk >= NBLK)) continue; // wave-uniform
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(dst + blk * 1024), 16,
                                                     goff[j], 0, 0, 0);
        }
#else
        (void)tb, (void)nrec, (void)goff, (void)dst, (void)first_blk;
#endif
    };
    // K tile t starts KSHIFT sub-tiles before V tile t; the rows of K tile 0 that would lie before
    // key 0 are not requested
    auto dma_k = [&](int t, int8_t *dst) __attribute__((always_inline)) {
        const int key0 = (t * NSUB - KSHIFT) * 32;
        dma_tile(Kp, p.ks[2], dma_goff_k, key0, key0 < 0 ? -key0 / RPB : 0, dst);
    };
    auto dma_v = [&](int t, int8_t *dst) __attribute__((always_inline)) { dma_tile(Vp, p.vs[2], dma_goff_v, t * BK, 0, dst); };

    dma_k(0, Ks0);
    dma_v(0, Vs0);
    dma_k(1, Ks1);

    auto lut_at = [&](int k) { return (uint32_t)k <= top ? (p.lut[k / 4] >> (8 * (k % 4))) & 0xffu : 0u; };
    // The clip points of classes 1 .. 3, per head: cap[n] = the first clipped distance whose index is >= 8 n, i.e. the
    // smallest x with 2 top x >= (16 n - 1) c_int (c_int where the table ends before index 8 n); ok[n]: that distance's
    // own index, the "probability 0" selector of the class, is exactly 8 n (thresholds below two per index step can
    // jump past it).  No integer division: the quotient comes from a double-precision estimate (the numerator is
    // below 2^36, so the estimate is off by one at most) and is corrected against the exact products.
    struct ClassCaps {
        int32_t cap[4];
        bool ok[4];
    };
    auto class_caps = [&](const HeadParams &hr) {
        ClassCaps cc;
        const double inv = __builtin_amdgcn_rcp((double)(2u * top));
        const int64_t den = 2 * (int64_t)top, c2 = 2 * (int64_t)hr.c_int;
        cc.cap[0] = hr.c_int;
        cc.ok[0] = false;
#pragma unroll
        for (int nn = 1; nn <= 3; ++nn) {
            cc.cap[nn] = hr.c_int;
            cc.ok[nn] = true;
            if (8 * nn <= (int)top) {
                const int64_t num = (int64_t)(16 * nn - 1) * hr.c_int;
                int64_t x = (int64_t)(uint32_t)((double)num * inv); // below c_int: 16 n - 1 < 2 top here
                if (den * x < num) ++x;
                if (den * x < num) ++x;
                if (x > 0 && den * (x - 1) >= num) --x;
                const int64_t at = den * x + hr.c_int; // 2 c_int (index of x) <= at < 2 c_int (index of x + 1)
                cc.ok[nn] = x <= hr.c_int && at >= 8 * nn * c2 && at < (8 * nn + 1) * c2;
                cc.cap[nn] = (int32_t)min(x, (int64_t)hr.c_int);
            }
        }
        return cc;
    };
    // ---- class of every row
    // class n = 1, 2, 3: S > max(510 LUT_hat[8 n], 510), the row needs n register pairs and no probability exceeds
    // 127; 4: the whole table in four register pairs, for any row sum, with the probabilities stored as P - 128
    // like the LDS tables (only when the table has exactly 2^5 entries, so that its last entry, which is 0 by
    // Eq. lut16, can stand for hidden keys); 5: the tables in LDS.
    auto row_class = [&](uint32_t s_row, const ClassCaps &cc) {
        int c = top == 31u ? 4 : 5;
#pragma unroll
        for (int nn = 3; nn >= 1; --nn)
            if (cc.ok[nn] && s_row > max(510u * lut_at(8 * nn), 510u)) c = nn;
        return c;
    };
    const int qw0 = q0 + 32 * wave;
    const int row = qw0 + n; // this lane's query row
    const bool valid = row >= rlo && row < rhi;
    // the wave's path: the largest class among its rows (0: general path); rows outside [rlo, rhi) are inert
    const ClassCaps caps = class_caps(M == IDX_ROW64 ? row_hp(row) : hp);
    const int my_cls = valid ? row_class((uint32_t)p.ws_row_sum[(int64_t)bh * LQ + (row - rlo)], caps) : 1;
    const int path = __any(my_cls == 5) ? 0 : __any(my_cls == 4) ? 4 : __any(my_cls == 3) ? 3 : __any(my_cls == 2) ? 2 : 1;

    // Q fragments: row `row`, bytes [32 kb + 16 h, +16)
    v4i qf[RB][KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[0][kb] = v4i{0, 0, 0, 0};
        if (valid) qf[0][kb] = *(const v4i *)(Qp + (int64_t)(row - rlo) * p.qs[2] + kb * 32 + h * 16);
    }

    // ---- per-row state from the first launch
    RowIndex<M> ri[RB];
    uint32_t sum[RB];
    const HeadParams hrow = M == IDX_ROW64 ? row_hp(row) : hp;
    {
        const int mx = valid ? p.ws_row_max[(int64_t)bh * LQ + (row - rlo)] : 0;
        sum[0] = valid ? (uint32_t)p.ws_row_sum[(int64_t)bh * LQ + (row - rlo)] : 0u;
        if (sum[0] == 0) sum[0] = 1; // only rows outside [rlo, rhi); never stored
        ri[0].init(hrow, mx, top);
        if (p.dbg_row_max && h == 0 && valid) p.dbg_row_max[(int64_t)bh * LQ + (row - rlo)] = mx;
        if (p.dbg_row_sum && h == 0 && valid) p.dbg_row_sum[(int64_t)bh * LQ + (row - rlo)] = (int32_t)sum[0];
    }

    // ---- register tables of the permute paths: tab[2 k], tab[2 k + 1] hold entries 8 k .. 8 k + 7 of
    // P_hat[idx] = round(255 LUT_hat[idx] / S); the clip of path n at the first distance of index 8 n
    RowIndex<M> rif[RB];
    uint32_t tab[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    rif[0] = ri[0];
    if (path != 0) {
        const int cap = path == 1 ? caps.cap[1] : (path == 2 ? caps.cap[2] : (path == 3 ? caps.cap[3] : hrow.c_int));
        rif[0].bound = ri[0].mx - cap;
        const float rs = __builtin_amdgcn_rcpf((float)(2u * sum[0]));
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            if (k < 8 * path) { // wave-uniform
                uint32_t q = prob_u8(lut_at(k), sum[0], rs);
                if (path == 4) q ^= 0x80u; // P - 128 as a byte; rows outside the problem: probability 0
                tab[k / 4] |= (valid ? q : (path == 4 ? 0x80u : 0u)) << (8 * (k % 4));
            }
        }
    }

    // Column sums of V over every key the steps below cover (keys up to the end of this query tile
    // under the causal mask, else all): the correction for feeding the probabilities to the signed
    // MFMA as P - 128.  A small kernel ahead of this one left the sums of each BQ-key chunk.
    if (tid < D) {
        const int32_t *cp = p.ws_colsum + (int64_t)(b * p.Hkv + kvh) * p.n_chunks * D + tid;
        const int nchunk = CAUSAL ? min(qt + 1, p.n_chunks) : p.n_chunks;
        int32_t acc = 0;
#pragma unroll 8
        for (int c = 0; c < nchunk; ++c) acc += cp[(int64_t)c * D];
        colsum[tid] = acc;
    }
    publish_tiles_barrier(); // LUT_hat, K tiles 0 and 1, V tile 0 are in LDS

    // per-row probability table of the general path: PT[idx] = round(255 * LUT_hat[idx] / sum) - 128 as a
    // byte; each lane of a row's pair computes half of the entries and stores them into both lanes' columns
    const uint32_t lane_off = (uint32_t)(4 * lane + wave);
    const uint32_t lane_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint8_t *)PT + lane_off;
    if (path == 0) {
        const uint8_t *lut_b = (const uint8_t *)lut_lds;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int kidx = 16 * h + j;
            const uint32_t e = lut_b[kidx];
            const uint32_t pr = prob_u8(e, sum[0], __builtin_amdgcn_rcpf((float)(2u * sum[0])));
            const uint8_t byte = (uint8_t)((pr ^ 0x80u) & 0xffu);
            PT[kidx * 256 + 4 * n + wave] = byte;
            PT[kidx * 256 + 4 * (n + 32) + wave] = byte;
        }
    }

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
    auto visible = [&](int key, int) { return key < L && (!CAUSAL || key <= row); };

    // ---- pipeline state
    v16i o[RB][CB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[rb][cb][i] = 0;
    v4i kf[KB], vf[CB];
    v4i pfA[RB], pfB[RB];      // MFMA operands of the probabilities of an even / odd sub-tile
    v16i sA[RB], sB[RB];       // raw scores of the sub-tile in flight / being accumulated
    uint32_t lA[NEL], lB[NEL]; // looked-up probability bytes (xor 0x80); only half a step's worth is live

    // Packs the looked-up bytes of scores [w0, w0 + EPS) (w = 16 rb + e) of sub-tile jp.
    auto pack = [&](auto masked_tag, int jp, const uint32_t (&l)[NEL], int w0, v4i (&pf)[RB]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int rb = w0 / 16, e0 = w0 % 16, g = e0 / 4;
        uint32_t bt[EPS];
#pragma unroll
        for (int r = 0; r < EPS; ++r) {
            bt[r] = l[w0 + r];
            if (MASKED) bt[r] = visible(32 * jp + acc_key(e0 + r, h), rb) ? bt[r] : 0x80u;
        }
        // byte permutes: two looked-up bytes into a pair, two pairs into the operand register
        const uint32_t pair = __builtin_amdgcn_perm(bt[1], bt[0], 0x0c0c0400u);
        if (EPS == 4) {
            const uint32_t pair2 = __builtin_amdgcn_perm(bt[3 % EPS], bt[2 % EPS], 0x0c0c0400u);
            pf[rb][g] = (int)__builtin_amdgcn_perm(pair2, pair, 0x05040100u);
        } else {
            pf[rb][g] = (e0 % 4 == 0) ? (int)pair : (int)__builtin_amdgcn_perm(pair, (uint32_t)pf[rb][g], 0x05040100u);
        }
    };

    // One pipeline step (see the head of the file).  sc: scores of sub-tile j; sn: receives the
    // scores of sub-tile j+1; lc / pfc: lookups and operands of sub-tile j; lp / pfp: of sub-tile j-1.
    // A score looked up after MFMA slot s is packed HALF slots later, so only half a step's lookups
    // are in flight and the packing never waits for what was just issued.  On entry kf holds the K
    // fragments of sub-tile j+1 and vf the V^T fragments of sub-tile j-1.
    uint32_t selw[RB]; // permute paths: index bytes of the operand register being assembled
    // Four probabilities from four packed index bytes s4 (each 0 .. 8 NP, where 8 NP is the clipped index)
    // and the row's NP register pairs.  lift(x) = x | ((x & 8) << 1) keeps 0..7 and turns 8..15 into
    // 24..31, so a lifted selector is 0..7 inside its pair and >= 16 (permute result 0xff) outside; the
    // last pair's selector is left so that the clipped index becomes 8, the sign of a byte below 128: 0.
    //   NP = 2:  A = lift(s): 0..7 | 24..31 | 16;    A ^ 24: 24..31 | 0..7 | 8
    //   NP = 3:  lift(s): 0..7 | 24..31 | 16..23 | 24;   lift(s ^ 8): 24..31 | 0..7 | 24..31 | 16;
    //            s ^ 16: 16..23 | 24..31 | 0..7 | 8
    auto lookup = [&](auto np_tag, uint32_t s4) __attribute__((always_inline)) {
        constexpr int NP = decltype(np_tag)::value;
        auto lift = [](uint32_t x) { const uint32_t t = x & 0x08080808u; return x | (t + t); };
        if (NP == 1) return __builtin_amdgcn_perm(tab[1], tab[0], s4);
        if (NP == 2) {
            const uint32_t sa = lift(s4);
            return __builtin_amdgcn_perm(tab[1], tab[0], sa) & __builtin_amdgcn_perm(tab[3], tab[2], sa ^ 0x18181818u);
        }
        if (NP == 3)
            return __builtin_amdgcn_perm(tab[1], tab[0], lift(s4)) & __builtin_amdgcn_perm(tab[3], tab[2], lift(s4 ^ 0x08080808u)) &
                   __builtin_amdgcn_perm(tab[5], tab[4], s4 ^ 0x10101010u);
        // NP = 4: every index is 0 .. 31 (hidden keys take 31, whose entry is probability 0, the byte 0x80 in this
        // path); pair k sees lift(s ^ 8 k), which is 0 .. 7 for its own indices and 16 .. 31 for all others
        return __builtin_amdgcn_perm(tab[1], tab[0], lift(s4)) & __builtin_amdgcn_perm(tab[3], tab[2], lift(s4 ^ 0x08080808u)) &
               __builtin_amdgcn_perm(tab[5], tab[4], lift(s4 ^ 0x10101010u)) & __builtin_amdgcn_perm(tab[7], tab[6], lift(s4 ^ 0x18181818u));
    };
    auto step = [&](auto masked_tag, auto path_tag, int j, const int8_t *Knext, const int8_t *Vcur, const v16i (&sc)[RB], v16i (&sn)[RB],
                    const uint32_t (&lp)[NEL], uint32_t (&lc)[NEL], v4i (&pfp)[RB], v4i (&pfc)[RB]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr int NP = decltype(path_tag)::value; // register pairs of the permute path; 0: tables in LDS
#pragma unroll
        for (int sl = 0; sl < NSLOT; ++sl) {
            if (sl < HALF) {
                const int kb = sl / RB, rb = sl % RB;
                if (kb == 0)
                    sn[rb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[0], qf[rb][0], v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, 0, 0, 0);
                else
                    sn[rb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[rb][kb], sn[rb], 0, 0, 0);
            } else {
                const int cb = (sl - HALF) / RB, rb = (sl - HALF) % RB;
                o[rb][cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[cb], pfp[rb], o[rb][cb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (NP != 0) {
                // index of each score (0 .. 8 NP after the short clip) as a byte: two byte permutes pair
                // them up, a third joins the pairs, and four probabilities come out of the row's table
                // registers.  IDX_TOP24: the index is the top byte of the scaled score and is picked up
                // there; the other schemes deliver it in the low byte.
                constexpr uint32_t PAIR = M == IDX_TOP24 ? 0x0c0c0703u : 0x0c0c0400u;
                constexpr uint32_t HID = NP == 4 ? 31u : (uint32_t)(8 * NP); // index that stands for a hidden key
                constexpr uint32_t CLIPPED = M == IDX_TOP24 ? HID << 24 : HID;
                uint32_t ivp = 0;
#pragma unroll
                for (int w = sl * EPS; w < (sl + 1) * EPS; ++w) {
                    const int rb = w / 16, e = w % 16;
                    const int c = max(sc[rb][e], rif[rb].bound);
                    uint32_t iv = M == IDX_TOP24 ? rif[rb].scaled(c) : rif[rb](c);
                    if (MASKED) iv = visible(32 * j + acc_key(e, h), rb) ? iv : CLIPPED; // also covers hidden keys above the row max
                    if (e % 2 == 0) {
                        ivp = iv;
                    } else {
                        const uint32_t pair = __builtin_amdgcn_perm(iv, ivp, PAIR);
                        if (e % 4 == 1) selw[rb] = pair;
                        else pfc[rb][e / 4] = (int)lookup(path_tag, __builtin_amdgcn_perm(pair, selw[rb], 0x05040100u));
                    }
                }
            } else {
                if (sl < HALF) pack(masked_tag, j - 1, lp, (sl + HALF) * EPS, pfp);
                else pack(masked_tag, j, lc, (sl - HALF) * EPS, pfc);
#pragma unroll
                for (int w = sl * EPS; w < (sl + 1) * EPS; ++w) {
                    const int rb = w / 16, e = w % 16;
                    // hidden keys may exceed the row max
                    const int c = MASKED ? min(max(sc[rb][e], ri[rb].bound), ri[rb].mx) : max(sc[rb][e], ri[rb].bound);
                    lc[w] = *(const __attribute__((address_space(3))) uint8_t *)(uintptr_t)ri[rb].row_addr(c, lane_base);
                }
            }
            if (sl == HALF - 1) read_kf(Knext, kf); // the scores' MFMAs have all issued
            if (sl == NSLOT - 1) read_vf(Vcur, vf);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One iteration = V tile T: the lookups of its NSUB sub-tiles, the scores of the NSUB sub-tiles
    // two further on (K tile T+1).  With PAR = T & 1: K tile T+2 replaces K tile T (read an iteration
    // ago) in Ks[PAR], V tile T+1 replaces V tile T-1 in Vs[PAR^1]; K tile T+1 is read from Ks[PAR^1]
    // and V tile T from Vs[PAR].
    auto iteration = [&](auto masked_tag, auto path_tag, int T, int8_t *Kdma, int8_t *Vdma, const int8_t *Krd, const int8_t *Vrd)
                         __attribute__((always_inline)) {
        if (T + 2 <= ntiles) dma_k(T + 2, Kdma);
        if (T + 1 < ntiles) dma_v(T + 1, Vdma);
#pragma unroll
        for (int u = 0; u < NSUB; u += 2) {
            step(masked_tag, path_tag, NSUB * T + u, Krd + u * SUB, Vrd + u * SUB, sA, sB, lB, lA, pfB, pfA);
            step(masked_tag, path_tag, NSUB * T + u + 1, Krd + (u + 1) * SUB, Vrd + (u + 1) * SUB, sB, sA, lA, lB, pfA, pfB);
        }
        publish_tiles_barrier(); // K tile T + 2 and V tile T + 1 have landed; every wave is done with tile T
    };

    // ---- prologue: scores of sub-tile 0, fragments of sub-tile 1 (the last two sub-tiles of K tile 0);
    // an empty "sub-tile -1"
    read_kf(Ks0 + KSHIFT * SUB, kf);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        sA[rb] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) sA[rb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[kb], qf[rb][kb], sA[rb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    read_kf(Ks0 + (KSHIFT + 1) * SUB, kf);
#pragma unroll
    for (int i = 0; i < NEL; ++i) lB[i] = 0; // operand bytes 0 = probability 128 - 128: adds nothing
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) vf[cb] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        pfA[rb] = v4i{0, 0, 0, 0};
        pfB[rb] = v4i{0, 0, 0, 0};
    }
    __syncthreads(); // every wave has read K tile 0 before iteration 0 overwrites it with K tile 2

    // Iterations whose sub-tiles are all fully visible to this wave need no masks (wave-uniform
    // count).  They run in pairs in a loop of their own, every buffer named statically (the compiler
    // then knows which direct-to-LDS load a fragment read depends on) and no branch inside the body;
    // the few remaining iterations take the masked code with the buffers chosen at run time.
    // Every wave of the workgroup passes the same number of barriers whichever path it takes: one per
    // iteration, ntiles in all.
    const int nfull_sub = CAUSAL ? min(L / 32, (qw0 + 1) / 32) : L / 32;
    const int nhot = min(nfull_sub / NSUB, ntiles);
    auto sweep = [&](auto path_tag) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(path_tag)::value != 0;
        int T = 0;
        for (; T + 2 <= nhot; T += 2) {
            iteration(std::false_type{}, path_tag, T, Ks0, Vs1, Ks1, Vs0);
            iteration(std::false_type{}, path_tag, T + 1, Ks1, Vs0, Ks0, Vs1);
        }
#pragma unroll 1
        for (; T < ntiles; ++T) {
            const bool odd = T & 1;
            iteration(std::true_type{}, path_tag, T, odd ? Ks1 : Ks0, odd ? Vs0 : Vs1, odd ? Ks0 : Ks1, odd ? Vs1 : Vs0);
        }
        // ---- drain: the last sub-tile's probabilities meet V (V^T fragments in vf); in the general path
        // the second half of its lookups (in lB) is packed first
        if (!FAST) {
#pragma unroll
            for (int sl = 0; sl < HALF; ++sl) pack(std::true_type{}, NSUB * ntiles - 1, lB, (sl + HALF) * EPS, pfB);
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) o[rb][cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[cb], pfB[rb], o[rb][cb], 0, 0, 0);
    };
    if (path == 1) sweep(std::integral_constant<int, 1>{});
    else if (path == 2) sweep(std::integral_constant<int, 2>{});
    else if (path == 3) sweep(std::integral_constant<int, 3>{});
    else if (path == 4) sweep(std::integral_constant<int, 4>{});
    else sweep(std::integral_constant<int, 0>{});

    // ================================================================= epilogue (Sec. 3.2: requantization)
    // (instantiated for the shift range and for the debug tap, so that the 64 values of a lane meet no branch)
    auto epilogue = [&](auto fast_tag, auto dbg_tag) __attribute__((always_inline)) {
        constexpr bool FAST = decltype(fast_tag)::value, DBG = decltype(dbg_tag)::value;
        int8_t *Op = p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)(row - rlo) * p.os[2];
        // the general path fed P - 128 to the signed MFMA: add 128 times the column sums of V back
        const int32_t cfac = (path == 0 || path == 4) ? 128 : 0;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch0 = cb * 32 + 8 * g + 4 * h;
                uint32_t packed = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int32_t acc = o[0][cb][4 * g + r] + cfac * colsum[ch0 + r];
                    if (DBG) p.dbg_acc[((int64_t)bh * LQ + (row - rlo)) * D + ch0 + r] = acc;
                    packed |= ((uint32_t)requant<FAST>(acc, hrow.rq_mult, hrow.rq_shift) & 0xffu) << (8 * r);
                }
                *(uint32_t *)(Op + ch0) = packed;
            }
        }
    };
    if (valid) {
        const bool fast = hrow.rq_shift >= 33;
        if (p.dbg_acc) {
            if (fast) epilogue(std::true_type{}, std::true_type{});
            else epilogue(std::false_type{}, std::true_type{});
        } else {
            if (fast) epilogue(std::true_type{}, std::false_type{});
            else epilogue(std::false_type{}, std::false_type{});
        }
    }
    };
    if constexpr (MODE == IDX_MIX) {
        if (hp.pad[0] == IDX_TOP24) body(std::integral_constant<int, IDX_TOP24>{}); // uniform for the workgroup
        else body(std::integral_constant<int, IDX_MULHI24>{});
    } else {
        body(std::integral_constant<int, MODE>{});
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
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_TOP24>), grid, block, 0, st, pf);
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_FP64>), grid, block, 0, st, pf);
        return (int)hipGetLastError();
    }
    if (idx_mode == IDX_MIX)
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_MIX>), grid, block, 0, st, p);
    else if (idx_mode == IDX_TOP24)
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_TOP24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_MAD24)
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_MAD24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_MULHI24)
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_MULHI24>), grid, block, 0, st, p);
    else if (idx_mode == IDX_FP32)
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_FP32>), grid, block, 0, st, p);
    else if (idx_mode == IDX_ROW64)
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_ROW64>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((sweep_c_kernel<D, RB, CAUSAL, IDX_FP64>), grid, block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

// 32 query rows per wave: p.n_qtiles must count tiles of 128 query rows, and the V chunk sums in
// p.ws_colsum must be over chunks of as many keys; p.ws_row_max / ws_row_sum filled.
int launch_sweep_c(const FwdParams &p, int d, int idx_mode, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (d == 64) return p.causal ? launch_mode<64, 1, true>(p, idx_mode, st) : launch_mode<64, 1, false>(p, idx_mode, st);
    if (d == 128) return p.causal ? launch_mode<128, 1, true>(p, idx_mode, st) : launch_mode<128, 1, false>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
