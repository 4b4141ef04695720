// Fused IntAttention forward for gfx950 (MI355X).
//
// One workgroup = 4 wavefronts = 128 query rows of one (batch, query head); each wavefront
// owns 32 query rows.  Keys/values stream through LDS in tiles of 32 keys.  Because
// IndexSoftmax (Sec. 3.1-3.2) needs the exact row maximum before any table index and the
// exact row sum before any probability, the key axis is swept three times, recomputing the
// INT8 score tile each time instead of ever storing the L x L matrix:
//   sweep A: S^T = K.Q^T (MFMA)            -> running row max
//   sweep B: S^T - max (MFMA accumulator starts at -max) -> clip, index, LUT_hat -> row sum
//            then the 2^b distinct probabilities of the row, P_hat = round(255 E/S), go to a
//            per-row table in LDS
//   sweep C: S^T again -> index -> per-row table -> 16 probability bytes per lane, which
//            are exactly one MFMA B operand of O^T += V^T.P^T; then requantize and store.
// Scores are produced transposed (keys x queries) so that each lane owns one query row:
// row max and row sum are in-lane plus one exchange between the two half-waves.
//
// The int8 MFMA is signed x signed while P_hat is unsigned (0..255).  The kernel feeds
// P_hat - 128 and adds 128 * (column sums of the V rows of every processed tile) at the end;
// hidden keys inside a processed tile carry P_hat = 0, i.e. the byte -128, so the correction
// is the plain column sum.  All intermediate magnitudes stay below 2^31 for L < 131072.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "params.h"

namespace intattn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;
constexpr int BQ = WAVES * 32; // query rows per workgroup
constexpr int BK = 32;         // keys per tile

template <int MODE>
__device__ __forceinline__ uint32_t index_map(uint32_t dclip, const HeadParams &hp, uint32_t top)
{
    if (MODE == IDX_MAD24) {
        return (__umul24(dclip, hp.idx_mul) + hp.idx_add) >> hp.idx_shift;
    } else {
        const uint64_t c = (uint64_t)(uint32_t)hp.c_int;
        return (uint32_t)((2ull * top * dclip + c) / (2ull * c));
    }
}

// Key index held in accumulator register i of a 32x32 MFMA result by a lane of half-wave h.
__device__ __forceinline__ int acc_key(int i, int h) { return 8 * (i >> 2) + 4 * h + (i & 3); }

template <int D, bool CAUSAL, int MODE>
__global__ __launch_bounds__(NT) void fwd_kernel(const FwdParams p)
{
    constexpr int KB = D / 32; // 32-wide blocks of the head dimension
    constexpr int CB = D / 32; // 32-wide blocks of output channels

    __shared__ __attribute__((aligned(16))) int8_t Ks[BK * D];  // [KB][32 keys][32 B]
    __shared__ __attribute__((aligned(16))) int8_t Vt[BK * D];  // [D channels][2 halves x 16 B]
    __shared__ uint32_t PT[WAVES][32 * 32];                      // [idx][row] per wave
    __shared__ uint32_t lut_lds[8];
    __shared__ int32_t cs_part[8][D];
    __shared__ int32_t colsum[D];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int nbh = p.B * p.Hq;
    const int bh = blockIdx.x % nbh;
    const int qt = p.n_qtiles - 1 - blockIdx.x / nbh; // long (late) causal tiles first
    const int b = bh / p.Hq, hq = bh % p.Hq, kvh = hq / p.group;
    const HeadParams hp = p.hp_table ? p.hp_table[hq] : p.hp0;
    const int L = p.L;
    const uint32_t top = (uint32_t)p.top;
    const uint32_t c_int = (uint32_t)hp.c_int;

    const int q0 = qt * BQ, qw0 = q0 + wave * 32, row = qw0 + n;
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    if (tid < 8) lut_lds[tid] = p.lut[tid];

    // Q fragment of this lane: row `row`, bytes [32 kb + 16 h, +16) of each 32-byte block.
    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (row < L) qf[kb] = *(const v4i *)(Qp + (int64_t)row * p.qs[2] + kb * 32 + h * 16);
    }

    const int kmax = CAUSAL ? min(L, q0 + BQ) : L;
    const int ntiles = (kmax + BK - 1) / BK;

    auto stage_k = [&](int t) {
        for (int c = tid; c < BK * (D / 16); c += NT) {
            const int key = c / (D / 16), ch = c % (D / 16);
            const int gk = t * BK + key;
            v4i val = v4i{0, 0, 0, 0};
            if (gk < L) val = *(const v4i *)(Kp + (int64_t)gk * p.ks[2] + ch * 16);
            *(v4i *)(Ks + (ch >> 1) * 1024 + key * 32 + (ch & 1) * 16) = val;
        }
    };

    auto qk_tile = [&](v16i s) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const v4i a = *(const v4i *)(Ks + kb * 1024 + n * 32 + h * 16);
            s = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qf[kb], s, 0, 0, 0);
        }
        return s;
    };

    // ---------------------------------------------------------------- sweep A: row max
    int mx = INT32_MIN;
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
        stage_k(t);
        __syncthreads();
        const int klo = t * BK;
        if (CAUSAL && klo > qw0 + 31) continue; // wave-uniform: tile hidden from all 32 rows
        v16i s = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        s = qk_tile(s);
        const bool need_mask = (klo + BK > L) || (CAUSAL && klo + BK - 1 > qw0);
        if (need_mask) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = klo + acc_key(i, h);
                const bool ok = key < L && (!CAUSAL || key <= row);
                if (ok) mx = max(mx, s[i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = max(mx, s[i]);
        }
    }
    mx = max(mx, __shfl_xor(mx, 32));

    // ---------------------------------------------------------------- sweep B: row sum of E_hat
    const uint8_t *lut_b = (const uint8_t *)lut_lds;
    uint32_t sum = 0;
    {
        v16i negm;
#pragma unroll
        for (int i = 0; i < 16; ++i) negm[i] = -mx;
        for (int t = 0; t < ntiles; ++t) {
            __syncthreads();
            stage_k(t);
            __syncthreads();
            const int klo = t * BK;
            if (CAUSAL && klo > qw0 + 31) continue;
            const v16i s = qk_tile(negm); // s[i] = A_hat - rowMax <= 0 for visible keys
            const bool need_mask = (klo + BK > L) || (CAUSAL && klo + BK - 1 > qw0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int nd = max(s[i], -(int)c_int);                // -min(Delta, c_int)
                if (need_mask) nd = min(nd, 0);                 // hidden keys may exceed the max
                const uint32_t idx = index_map<MODE>((uint32_t)(-nd), hp, top);
                uint32_t e = lut_b[idx];
                if (need_mask) {
                    const int key = klo + acc_key(i, h);
                    const bool ok = key < L && (!CAUSAL || key <= row);
                    e = ok ? e : 0u;
                }
                sum += e;
            }
        }
    }
    sum += __shfl_xor(sum, 32);
    if (sum == 0) sum = 1; // only rows beyond L; never stored

    // per-row probability table: PT[idx] = round(255 * LUT_hat[idx] / sum) - 128 as a byte
    {
        uint32_t *pt = PT[wave];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int kidx = 16 * h + j;
            const uint32_t e = lut_b[kidx];
            const uint32_t pr = (510u * e + sum) / (2u * sum);
            pt[kidx * 32 + n] = (pr ^ 0x80u) & 0xffu;
        }
    }
    if (p.dbg_row_max && h == 0 && row < L) p.dbg_row_max[(int64_t)bh * L + row] = mx;
    if (p.dbg_row_sum && h == 0 && row < L) p.dbg_row_sum[(int64_t)bh * L + row] = (int32_t)sum;

    // ---------------------------------------------------------------- sweep C: P_hat and P_hat.V_hat
    v16i o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0;

    int32_t cs[4] = {0, 0, 0, 0}; // column sums of V for this thread's 4 channels / key group
    const int vG = tid / (D / 4), vcg = tid % (D / 4); // key group of 4, channel group of 4
    const bool v_active = tid < 8 * (D / 4);

    {
        v16i negm;
#pragma unroll
        for (int i = 0; i < 16; ++i) negm[i] = -mx;
        const uint32_t *pt = PT[wave];
        for (int t = 0; t < ntiles; ++t) {
            __syncthreads();
            stage_k(t);
            if (v_active) {
                // 4 keys x 4 channels -> transposed: one dword per channel holding 4 keys
                uint32_t w[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int gk = t * BK + 4 * vG + r;
                    w[r] = 0;
                    if (gk < L) w[r] = *(const uint32_t *)(Vp + (int64_t)gk * p.vs[2] + 4 * vcg);
                }
                const int slot_dw = 4 * (vG & 1) + (vG >> 1); // key 8g+4h+r -> byte 16h+4g+r
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t ov = ((w[0] >> (8 * c)) & 0xffu) | (((w[1] >> (8 * c)) & 0xffu) << 8) |
                                        (((w[2] >> (8 * c)) & 0xffu) << 16) | (((w[3] >> (8 * c)) & 0xffu) << 24);
                    *(uint32_t *)(Vt + (4 * vcg + c) * 32 + slot_dw * 4) = ov;
                    cs[c] += (int)(int8_t)(ov & 0xff) + (int)(int8_t)((ov >> 8) & 0xff) +
                             (int)(int8_t)((ov >> 16) & 0xff) + (int)(int8_t)(ov >> 24);
                }
            }
            __syncthreads();
            const int klo = t * BK;
            v4i pf;
            if (CAUSAL && klo > qw0 + 31) {
                pf = v4i{(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
            } else {
                const v16i s = qk_tile(negm);
                const bool need_mask = (klo + BK > L) || (CAUSAL && klo + BK - 1 > qw0);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t packed = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 4 * g + r;
                        int nd = max(s[i], -(int)c_int);
                        if (need_mask) nd = min(nd, 0);
                        const uint32_t idx = index_map<MODE>((uint32_t)(-nd), hp, top);
                        uint32_t pb = pt[idx * 32 + n];
                        if (need_mask) {
                            const int key = klo + acc_key(i, h);
                            const bool ok = key < L && (!CAUSAL || key <= row);
                            pb = ok ? pb : 0x80u;
                        }
                        packed |= pb << (8 * r);
                    }
                    pf[g] = (int)packed;
                }
            }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const v4i a = *(const v4i *)(Vt + (cb * 32 + n) * 32 + h * 16);
                o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, pf, o[cb], 0, 0, 0);
            }
        }
    }

    // ---------------------------------------------------------------- epilogue
    __syncthreads();
    if (v_active) {
#pragma unroll
        for (int c = 0; c < 4; ++c) cs_part[vG][4 * vcg + c] = cs[c];
    }
    __syncthreads();
    if (tid < D) {
        int32_t a = 0;
#pragma unroll
        for (int g = 0; g < 8; ++g) a += cs_part[g][tid];
        colsum[tid] = a;
    }
    __syncthreads();

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
int launch_mode(const FwdParams &p, int idx_mode, hipStream_t st)
{
    const dim3 grid((unsigned)(p.n_qtiles * p.B * p.Hq)), block(NT);
    if (idx_mode == IDX_MAD24)
        hipLaunchKernelGGL((fwd_kernel<D, CAUSAL, IDX_MAD24>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((fwd_kernel<D, CAUSAL, IDX_DIV>), grid, block, 0, st, p);
    return (int)hipGetLastError();
}

} // namespace

int fwd_rows_per_block(int /*variant*/) { return BQ; }

int launch_fwd(const FwdParams &p, int d, int idx_mode, int /*variant*/, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (d == 64) return p.causal ? launch_mode<64, true>(p, idx_mode, st) : launch_mode<64, false>(p, idx_mode, st);
    if (d == 128) return p.causal ? launch_mode<128, true>(p, idx_mode, st) : launch_mode<128, false>(p, idx_mode, st);
    return (int)hipErrorInvalidValue;
}

} // namespace intattn
