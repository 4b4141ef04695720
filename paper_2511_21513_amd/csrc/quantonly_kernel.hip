// In-run comparator: the conventional INT8 attention pipeline the paper calls "Quant-Only"
// (Sec. 2.2, "Emerging Bottleneck in Quantized Attention Pipelines"): INT8 Q.K^T into INT32,
// dequantize to fp32 with alpha = s_Q s_K / sqrt(d), fp32 softmax, requantize the
// probabilities to signed INT8 scaled by 127 (Sec. 3.2 describes that convention), INT8 P.V
// into INT32, and requantize the output with the same s_O as the integer path.
//
// To make the comparison fair it is fused and tiled exactly like the integer kernel (same
// workgroup shape, same LDS tile layout, same MFMA formulation with one query row per lane),
// and uses the single-sweep online softmax that a floating-point pipeline allows: the
// running row maximum rescales the fp32 output accumulator, so K and V are read once.
// Probabilities are quantized per 64-key tile relative to the running maximum.
// Its result approximates fp softmax attention; it is not compared bit-for-bit with anything.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace {

constexpr int WAVES = 4;
constexpr int NT = WAVES * 64;
constexpr int BQ = WAVES * 32;
constexpr int BK = 64;

template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT, 2) void quantonly_kernel(const FwdParams p)
{
    constexpr int KB = D / 32;
    constexpr int CB = D / 32;
    constexpr int TILE = BK * D;
    constexpr int CPT = TILE / 16 / NT;
    static_assert(CPT >= 1 && CPT * 16 * NT == TILE, "tile must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) int8_t Ks[2][TILE];
    __shared__ __attribute__((aligned(16))) int8_t Vs[2][TILE];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n = lane & 31, h = lane >> 5;
    const WorkItem wi = fwd_work_item(p, (int)blockIdx.x);
    if (!wi.valid) return;
    const int b = wi.b, hq = wi.hq, kvh = wi.kvh, qt = wi.qt;
    const int L = p.L;
    const float alpha = p.alpha_table ? p.alpha_table[hq] : p.alpha0;
    const float sv_over_so = p.svso_table ? p.svso_table[hq] : p.sv_over_so0;
    const float sc = alpha * 1.44269504088896340736f; // logits in units of log2

    const int q0 = qt * BQ, qw0 = q0 + wave * 32, row = qw0 + n;
    const int8_t *Qp = p.q + (int64_t)b * p.qs[0] + (int64_t)hq * p.qs[1];
    const int8_t *Kp = p.k + (int64_t)b * p.ks[0] + (int64_t)kvh * p.ks[1];
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];

    v4i qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        qf[kb] = v4i{0, 0, 0, 0};
        if (row < L) qf[kb] = *(const v4i *)(Qp + (int64_t)row * p.qs[2] + kb * 32 + h * 16);
    }

    const int kmax = CAUSAL ? min(L, q0 + BQ) : L;
    const int ntiles = (kmax + BK - 1) / BK;

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
        const int8_t *tb = base + (int64_t)t * BK * stride;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const uint32_t off = (t * BK + st_key[j] < L) ? (uint32_t)goff[j] : 0u;
            st[j] = *(const v4i *)(tb + off);
        }
    };
    auto store_tile = [&](int8_t *dst, const int (&loff)[CPT], int t, v4i (&st)[CPT]) {
        if ((t + 1) * BK > L) {
#pragma unroll
            for (int j = 0; j < CPT; ++j)
                if (t * BK + st_key[j] >= L) st[j] = v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < CPT; ++j) *(v4i *)(dst + loff[j]) = st[j];
    };
    auto visible = [&](int key) { return key < L && (!CAUSAL || key <= row); };

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

    float o[CB][16];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[cb][i] = 0.f;
    float m_run = -1.0e30f; // running row maximum, log2 units
    float l_run = 0.f;      // this lane's share of the running denominator

    load_tile(Kp, p.ks[2], st_goff_k, 0, stage_k);
    load_tile(Vp, p.vs[2], st_goff_v, 0, stage_v);
    store_tile(Ks[0], st_lds_k, 0, stage_k);
    store_tile(Vs[0], st_lds_v, 0, stage_v);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) {
            load_tile(Kp, p.ks[2], st_goff_k, t + 1, stage_k);
            load_tile(Vp, p.vs[2], st_goff_v, t + 1, stage_v);
        }
        if (!(CAUSAL && t * BK > qw0 + 31)) { // tile not wholly hidden from this wave
            v16i s[2];
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[st][i] = 0;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const int key = 32 * st + n;
                    const v4i a = *(const v4i *)(Ks[buf] + key * D + (((2 * kb + h) ^ swz_k<D>(key)) << 4));
                    s[st] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qf[kb], s[st], 0, 0, 0);
                }
            }
            const bool full = (t + 1) * BK <= L && (!CAUSAL || (t + 1) * BK - 1 <= qw0);
            // dequantize (Eq. logit-scale) and take the tile's row maximum
            float x[2][16];
            float tmax = -1.0e30f;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float v = (float)s[st][i] * sc;
                    if (!full && !visible(t * BK + 32 * st + acc_key(i, h))) v = -1.0e30f;
                    x[st][i] = v;
                    tmax = fmaxf(tmax, v);
                }
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float m_new = fmaxf(m_run, tmax);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            // fp32 softmax numerators, requantized to signed INT8 scaled by 127
            v4i pf[2];
            float psum = 0.f;
#pragma unroll
            for (int st = 0; st < 2; ++st) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t packed = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float pr = __builtin_amdgcn_exp2f(x[st][4 * g + r] - m_new);
                        psum += pr;
                        packed |= (uint32_t)__float2int_rn(pr * 127.0f) << (8 * r);
                    }
                    pf[st][g] = (int)packed;
                }
            }
            l_run = l_run * corr + psum;
            // INT8 P.V for this tile, then fold into the rescaled fp32 accumulator
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                v16i ot;
#pragma unroll
                for (int i = 0; i < 16; ++i) ot[i] = 0;
                ot = __builtin_amdgcn_mfma_i32_32x32x32_i8(vt_frag(Vs[buf], 0, cb), pf[0], ot, 0, 0, 0);
                ot = __builtin_amdgcn_mfma_i32_32x32x32_i8(vt_frag(Vs[buf], 1, cb), pf[1], ot, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 16; ++i) o[cb][i] = o[cb][i] * corr + (float)ot[i];
            }
        }
        if (t + 1 < ntiles) {
            store_tile(Ks[buf ^ 1], st_lds_k, t + 1, stage_k);
            store_tile(Vs[buf ^ 1], st_lds_v, t + 1, stage_v);
        }
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (row < L) {
        // O = s_V * P.V_hat (Eq. pv-link) with P = P_int8 / 127; output in units of s_O
        const float scale = sv_over_so / (127.0f * l_tot);
        int8_t *Op = p.out + (int64_t)b * p.os[0] + (int64_t)hq * p.os[1] + (int64_t)row * p.os[2];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch0 = cb * 32 + 8 * g + 4 * h;
                uint32_t packed = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    int v = __float2int_rn(o[cb][4 * g + r] * scale);
                    v = v > 127 ? 127 : (v < -127 ? -127 : v);
                    packed |= ((uint32_t)v & 0xffu) << (8 * r);
                }
                *(uint32_t *)(Op + ch0) = packed;
            }
        }
    }
}

} // namespace

int launch_quantonly(const FwdParams &p_in, int d, int /*variant*/, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    FwdParams p = p_in;
    p.group_batch = fwd_group_batch(p.B, p.Hkv, 2 * (int64_t)p.Lk * d); // the same workgroup order as the integer path
    const dim3 grid((unsigned)fwd_grid_size(p.B, p.Hq, p.Hkv, p.n_qtiles)), block(NT);
    if (d == 64) {
        if (p.causal) hipLaunchKernelGGL((quantonly_kernel<64, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((quantonly_kernel<64, false>), grid, block, 0, st, p);
    } else if (d == 128) {
        if (p.causal) hipLaunchKernelGGL((quantonly_kernel<128, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((quantonly_kernel<128, false>), grid, block, 0, st, p);
    } else {
        return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

} // namespace intattn
