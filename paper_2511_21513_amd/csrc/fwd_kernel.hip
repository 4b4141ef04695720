// Host side of the forward launches: the kernel variants, the small kernel that sums V over chunks
// of keys, and the order of the launches of one forward.  The forward kernel template itself is in
// fwd_kernel_impl.h and is instantiated in fwd_single.hip (all three sweeps in one launch) and
// fwd_split.hip (sweeps A+B, and sweep C, as launches of their own).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernel_common.h"
#include "params.h"

namespace intattn {

namespace fwdk {
// instantiated explicitly in fwd_single.hip / fwd_split.hip
template <int RB, int KT, int PH>
int launch_shape(const FwdParams &p, int d, int idx_mode, hipStream_t st);
} // namespace fwdk
using fwdk::launch_shape;

namespace {

// Sums of V over each chunk of `chunk` consecutive keys, per (batch, KV head) and channel:
// out[((b * Hkv + kvh) * n_chunks + c) * D + ch].  Keys past Lk do not count.  The forward kernel
// adds up the chunks its tiles cover.
template <int D>
__global__ __launch_bounds__(256) void colsum_kernel(const FwdParams p, int chunk)
{
    constexpr int G = D / 16;   // 16-byte column groups of a key row
    constexpr int KL = 256 / G; // key lanes
    __shared__ int32_t red[KL][D + 1];
    const int tid = threadIdx.x, c16 = tid % G, kl = tid / G;
    const int c = blockIdx.x % p.n_chunks, bk = blockIdx.x / p.n_chunks, kvh = bk % p.Hkv, b = bk / p.Hkv;
    const int8_t *Vp = p.v + (int64_t)b * p.vs[0] + (int64_t)kvh * p.vs[1];
    int32_t acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0;
    const int kend = min(p.Lk, (c + 1) * chunk);
    for (int key = c * chunk + kl; key < kend; key += KL) {
        const v4i x = *(const v4i *)(Vp + (int64_t)key * p.vs[2] + c16 * 16);
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] += (int32_t)(int8_t)((uint32_t)x[i / 4] >> (8 * (i % 4)));
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) red[kl][c16 * 16 + i] = acc[i];
    __syncthreads();
    if (tid < D) {
        int32_t t = 0;
        for (int j = 0; j < KL; ++j) t += red[j][tid];
        p.ws_colsum[((int64_t)bk * p.n_chunks + c) * D + tid] = t;
    }
}

int launch_colsum(const FwdParams &p, int d, int chunk, hipStream_t st)
{
    const dim3 grid((unsigned)(p.B * p.Hkv * p.n_chunks)), block(256);
    if (d == 64) hipLaunchKernelGGL(colsum_kernel<64>, grid, block, 0, st, p, chunk);
    else if (d == 128) hipLaunchKernelGGL(colsum_kernel<128>, grid, block, 0, st, p, chunk);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

} // namespace

// Kernel variants (0 = automatic choice; the others are tuning knobs, all bit-identical):
//   1  one launch, 32 query rows per wave, 64-key tiles     2  one launch, 64 rows per wave
//   3  one launch, a workgroup per 32 query rows with the keys split over its four waves (fwd_splitk.hip)
//   4  two launches: sweeps A+B (64 rows per wave), then sweep C (32 rows per wave), phase-ordered kernels
//   5  as 4 with the software-pipelined sweep C kernel
//   9, 10  the split-key kernels of decode_kernel.hip (one launch / four launches) whenever the shape allows them, else as 0
// Automatic choice among the tiled kernels, by measurement on shapes from 8 x 12 x 197 to 2 x 32 x 4096 (W = workgroups
// of 128 query rows): W >= 1024 fills the chip with the two-launch path (variant 5), short rows excepted; up to 256 the 128-row kernels
// leave most SIMDs with one long-running wave and the split-key single launch (variant 3) is 1.1 to 2.3 times faster;
// in between variant 3 still wins at d = 64 on long rows, otherwise variant 1 (at d = 128 the four waves of variant 3
// each stream their own K fragments from L2, which costs more than the better fill gains).
int fwd_choose_variant(int variant, int B, int Hq, int L, int Lk, int d, int causal)
{
    if (variant != 0 && variant != 9 && variant != 10) return variant;
    const int nt = (L + 127) / 128;
    const int64_t workgroups = (int64_t)B * Hq * nt;
    // Short key runs (at most three key tiles per query tile on average: up to Lk = 384, or L = Lk = 640 under the
    // causal mask): one launch, which stages K once, beats two (c2 at batch 512: 0.29 against 0.37 ms).
    const int kt2 = causal ? 2 * ((Lk - L + 127) / 128) + nt + 1 : 2 * ((Lk + 127) / 128); // twice the average
    if (workgroups >= 1024) return kt2 <= 6 ? 1 : 5;
    if (workgroups <= 256) return 3;
    return (d == 64 && L >= 1024) ? 3 : 1;
}
bool fwd_variant_known(int variant) { return variant == 0 || (variant >= 1 && variant <= 5) || variant == 9 || variant == 10; }
int fwd_rows_per_block(int variant) { return variant == 2 ? 256 : (variant == 3 ? 32 : 128); }

int launch_fwd(const FwdParams &p_in, int d, int idx_mode, int variant, int stage, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    FwdParams p = p_in;
    const int64_t k_bytes = (int64_t)p.Lk * d; // K of one (batch, KV head) group; V is as large
    p.group_batch = fwd_group_batch(p.B, p.Hkv, 2 * k_bytes); // kernels that stream K and V
    const bool two_launches = variant == 4 || variant == 5;
    if (stage != 0 && !two_launches) return (int)hipErrorNotSupported;
    // all launches go to the same stream: V chunk sums first, then the sweeps
    int e = 0;
    if (variant == 3) {
        return launch_fwd_splitk(p, d, idx_mode, stream); // sums V itself
    }
    if (!two_launches && p.Lk <= 512) {
        // short key sequences: the single-launch kernels sum V themselves (one launch less)
        FwdParams ps = p;
        ps.ws_colsum = nullptr;
        if (variant == 2) return launch_shape<2, 2, 0>(ps, d, idx_mode, st);
        return launch_shape<1, 2, 0>(ps, d, idx_mode, st);
    }
    if (stage != 2) e = launch_colsum(p, d, fwd_rows_per_block(variant), st);
    if (e != 0) return e;
    if (variant == 2) return launch_shape<2, 2, 0>(p, d, idx_mode, st);
    if (two_launches) {
        // sweeps A+B leave row max and row sum in the workspace for sweep C
        if (stage != 2) {
            FwdParams pab = p;
            pab.n_qtiles = fwd_row_tiles(p.row_lo, p.L, 256); // 64 query rows per wave in the first launch
            pab.group_batch = fwd_group_batch(p.B, p.Hkv, k_bytes); // streams K only
            e = launch_shape<2, 2, 1>(pab, d, idx_mode, st);
            if (e != 0 || stage == 1) return e;
        }
        if (variant == 4) return launch_shape<1, 2, 2>(p, d, idx_mode, st);
        if (p.hp_table_c && idx_mode == IDX_MULHI24) {
            // most heads have top-byte constants, which cost sweep C one vector instruction per score less
            FwdParams pc = p;
            pc.hp_table = p.hp_table_c;
            return launch_sweep_c(pc, d, IDX_MIX, stream);
        }
        return launch_sweep_c(p, d, idx_mode, stream);
    }
    return launch_shape<1, 2, 0>(p, d, idx_mode, st);
}

} // namespace intattn
