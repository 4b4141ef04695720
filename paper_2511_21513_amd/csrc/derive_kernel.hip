// Per-head kernel parameters from scales that live in DEVICE memory (as the dynamic quantizer
// leaves them), so that quantizer and attention follow each other on a stream without the host
// reading anything back:
//   c_int = round(c * sqrt(d) / (s_Q s_K))                    (Sec. 3.1, Eq. clipping_thr)
//   (M, sh) with M * 2^-sh ~ s_V / (255 s_O), M in [2^30, 2^31)   (output requantization)
//   constants of an exact index map idx = round(x * top / c_int)  (Sec. 3.1, index map): the 24-bit
//   multiply-add whose top byte is the index where it exists, else the fp64 map
// The arithmetic is the host's, operation for operation, in IEEE double: products, quotients,
// floor, frexp and the fma are exactly rounded on the GPU as on the CPU, and sqrt(d) comes from the
// host.  One wave per query head, one check point of the index map per lane.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "params.h"

namespace intattn {

namespace {

__device__ __forceinline__ bool good_scale(float s) { return s > 0.0f && s < __builtin_inff(); } // false for NaN

__device__ __forceinline__ uint32_t exact_index(uint64_t x, uint64_t c_int, uint64_t top)
{
    return (uint32_t)((2 * top * x + c_int) / (2 * c_int));
}

// c_int (capped at 2^30: beyond 62 * 2 * 128*128*128 every index is 0 anyway) and the requantization
// multiplier of one parameter set; false (and harmless values) when a scale is unusable.
__device__ __forceinline__ bool derive_scalars(float sq, float sk, float sv, float so, double clip, double sqrt_d, HeadParams &hp)
{
    hp.pad[0] = IDX_FP64;
    hp.pad[1] = 0;
    bool ok = good_scale(sq) && good_scale(sk) && good_scale(sv) && good_scale(so);
    double c = 1.0;
    if (ok) {
        const double alpha = ((double)sq * (double)sk) / sqrt_d;
        c = __builtin_floor(clip / alpha + 0.5);
        if (!(c >= 1.0)) c = 1.0;
        if (c > 1073741824.0) c = 1073741824.0;
    }
    hp.c_int = (int32_t)c;
    // unusable scales: multiplier 0, i.e. the head's output is all zeros (and its status word is set)
    hp.rq_mult = 0;
    hp.rq_shift = 31;
    if (ok) {
        const double r = (double)sv / (255.0 * (double)so);
        int e = 0;
        const double m = __builtin_frexp(r, &e);
        long long M = __builtin_llround(m * 2147483648.0);
        if (M == 2147483648LL) {
            M = 1073741824LL;
            e += 1;
        }
        const int sh = 31 - e;
        if (!(r > 0.0) || sh < 1 || sh > 62) ok = false;
        else {
            hp.rq_mult = (int32_t)M;
            hp.rq_shift = sh;
        }
    }
    return ok;
}

// the fp64 index map's factor for c_int: the bits of -(the double after top / c_int), low word in
// idx_mul, high word in idx_add
__device__ __forceinline__ uint64_t set_fp64_factor(HeadParams &hp, uint32_t top)
{
    const uint64_t bits = (uint64_t)__double_as_longlong((double)top / (double)(uint32_t)hp.c_int) + 1ull;
    const uint64_t neg = bits ^ 0x8000000000000000ull;
    hp.idx_mul = (uint32_t)neg;
    hp.idx_add = (uint32_t)(neg >> 32);
    hp.idx_shift = 0;
    return bits;
}

// One wave per query head.  Lane l computes two check points x of the index map (numbers l and l + 64):
// x = 0, x = c_int, and both sides of each of the (at most 63) steps of the exact map; every map in
// question is a monotone step function, so agreement at these points is agreement on all of [0, c_int].
// The points go to LDS; then every lane tests one candidate multiplier of the top-byte scheme against
// all of them (two rounds of 64 candidates at most), so the search costs the same few microseconds
// whether or not constants exist.
__global__ __launch_bounds__(64) void derive_kernel(const DeriveParams dp)
{
    __shared__ uint32_t px[128], pk[128];
    const int h = blockIdx.x, lane = threadIdx.x;
    const int si = dp.per_head ? h : 0;
    const int kv = dp.per_head ? h / dp.group : 0;
    const float sq = dp.scale_q[si], sk = dp.scale_k[kv], sv = dp.scale_v[kv];
    const float so = dp.scale_out ? dp.scale_out[si] : sv;
    HeadParams hp;
    bool ok = derive_scalars(sq, sk, sv, so, dp.clip, dp.sqrt_d, hp);

    // this lane's check points
    const uint32_t c_int = (uint32_t)hp.c_int, top = (uint32_t)dp.top;
    uint32_t x[2], want[2];
    bool have[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int id = lane + 64 * q;
        x[q] = id == 0 ? 0u : c_int;
        have[q] = id < 2;
        if (id >= 2) {
            const uint64_t k = (uint64_t)((id - 2) >> 1) + 1;
            const uint64_t t = ((2 * k - 1) * (uint64_t)c_int + 2ull * top - 1) / (2ull * top); // first x whose index is >= k
            const uint32_t below = (uint32_t)(id & 1);
            have[q] = k <= top && t <= c_int && t >= below;
            x[q] = (uint32_t)t - below;
        }
        if (!have[q]) x[q] = 0u; // a second copy of the point x = 0
        want[q] = exact_index(x[q], c_int, top);
        px[id] = x[q];
        pk[id] = want[q];
    }
    __syncthreads();

    // (x * mul + add) >> 24 with a 23-bit multiplier (the host's find_top24, candidate for candidate):
    // a check point with exact index k confines add to [k 2^24 - x mul, (k + 1) 2^24 - 1 - x mul];
    // the first multiplier around top 2^24 / c_int whose intervals intersect is taken
    bool found = false;
    if (ok && c_int < (1u << 23)) { // wave-uniform
        const long long m0 = (long long)(((unsigned long long)top << 24) / c_int);
        for (int round = 0; round < 2 && !found; ++round) {
            const int cand = lane + 64 * round;
            const long long dm = cand >> 1, mul = (cand & 1) ? m0 - dm : m0 + 1 + dm;
            const bool valid = cand < 80 && mul >= 1 && mul < (1ll << 23);
            long long lo = 0, hi = valid ? (1ll << 31) - 1 - (long long)c_int * mul : -1;
            if (valid) {
                for (int i = 0; i < 128; ++i) {
                    const long long xm = (long long)px[i] * mul, k = (long long)pk[i];
                    lo = max(lo, (k << 24) - xm);
                    hi = min(hi, ((k + 1) << 24) - 1 - xm);
                }
            }
            const unsigned long long good = __ballot(lo <= hi);
            if (good != 0ull) {
                const int src = __builtin_ctzll(good); // the first candidate in the host's order
                const long long mul_s = __shfl(mul, src), lo_s = __shfl(lo, src), hi_s = __shfl(hi, src);
                found = true;
                hp.pad[0] = IDX_TOP24;
                hp.idx_mul = (uint32_t)(-(int32_t)mul_s);
                hp.idx_add = (uint32_t)(lo_s + (hi_s - lo_s) / 2);
                hp.idx_shift = 24;
            }
        }
    }
    if (!found) {
        // fp64 with r the double after top / c_int: exact for every c_int (the excess of r is under
        // two units in the last place and the fma rounds once, monotonically; values of
        // x*top/c_int + 1/2 that are not integers stay 1/(2 c_int) away from the next integer)
        const uint64_t bits = (uint64_t)__double_as_longlong((double)top / (double)c_int) + 1ull;
        const double r = __longlong_as_double((long long)bits);
        bool match = true;
#pragma unroll
        for (int q = 0; q < 2; ++q)
            if (have[q] && (uint32_t)(int)__builtin_fma(-(double)x[q], -r, 0.5) != want[q]) match = false;
        if (!__all(match)) ok = false;
        const uint64_t neg = bits ^ 0x8000000000000000ull;
        hp.pad[0] = IDX_FP64;
        hp.idx_mul = (uint32_t)neg;
        hp.idx_add = (uint32_t)(neg >> 32);
        hp.idx_shift = 0;
    }
    if (!ok) hp.rq_mult = 0; // (the fp64 check cannot fail; kept as the last line of defence)
    if (lane == 0) {
        dp.hp_table[h] = hp;
        dp.status[h] = ok ? 0 : 1;
    }
}

// All heads of a call run one index scheme: a launch that serves only some head indices leaves most of
// the chip idle, because the workgroups of a head index share an XCD.  If any head lacks top-byte
// constants, every head takes the fp64 map (exact for every threshold).  One wave.
__global__ __launch_bounds__(64) void unify_schemes_kernel(HeadParams *table, int n_heads, uint32_t top)
{
    bool mixed = false;
    for (int h = threadIdx.x; h < n_heads; h += 64) mixed |= table[h].pad[0] != IDX_TOP24;
    if (!__any(mixed)) return;
    for (int h = threadIdx.x; h < n_heads; h += 64) {
        HeadParams hp = table[h];
        if (hp.pad[0] == IDX_TOP24) {
            hp.pad[0] = IDX_FP64;
            set_fp64_factor(hp, top);
            table[h] = hp;
        }
    }
}

// Parameters per block of q_block query rows (finer quantization groups over the query rows,
// Sec. 3.3): one thread per (batch, head, block); scale_q / scale_out hold one value per block,
// scale_k / scale_v one per KV head.  Every block takes the fp64 index map, which is exact for
// every c_int without a search.
__global__ __launch_bounds__(256) void derive_rows_kernel(const DeriveParams dp)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= dp.n_entries) return;
    const int hq = (int)((e / dp.n_rowblk) % dp.Hq), kv = hq / dp.group;
    // with groups over the key axis too (n_kentries > 0) the key scales are checked by a kernel of their own
    // and c_int is formed per logit in the forward kernel: only the requantization is taken from here
    const float sq = dp.scale_q[e], sk = dp.n_kentries > 0 ? 1.0f : dp.scale_k[kv], sv = dp.scale_v[kv];
    const float so = dp.scale_out ? dp.scale_out[e] : sv;
    HeadParams hp;
    const bool ok = derive_scalars(sq, sk, sv, so, dp.clip, dp.sqrt_d, hp);
    set_fp64_factor(hp, (uint32_t)dp.top);
    dp.row_table[e] = hp;
    if (!ok) dp.status[hq] = 1; // every writer stores the same value
}

// Scales per block of keys, [B * Hkv][n_kblk]: an unusable one marks every query head of its KV head.
__global__ __launch_bounds__(256) void check_key_scales_kernel(const DeriveParams dp)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= dp.n_kentries) return;
    if (good_scale(dp.scale_k[e])) return;
    const int kv = (int)((e / dp.n_kblk) % dp.Hkv);
    for (int g = 0; g < dp.group; ++g) dp.status[kv * dp.group + g] = 1; // every writer stores the same value
}

__global__ __launch_bounds__(256) void zero_status_kernel(int32_t *status, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) status[i] = 0;
}

} // namespace

int launch_derive_rows(const DeriveParams &dp, void *stream)
{
    hipLaunchKernelGGL(zero_status_kernel, dim3((unsigned)((dp.Hq + 255) / 256)), dim3(256), 0, (hipStream_t)stream, dp.status, dp.Hq);
    hipLaunchKernelGGL(derive_rows_kernel, dim3((unsigned)((dp.n_entries + 255) / 256)), dim3(256), 0, (hipStream_t)stream, dp);
    return (int)hipGetLastError();
}

int launch_derive_groups(const DeriveParams &dp, void *stream)
{
    const int e = launch_derive_rows(dp, stream);
    if (e != 0) return e;
    hipLaunchKernelGGL(check_key_scales_kernel, dim3((unsigned)((dp.n_kentries + 255) / 256)), dim3(256), 0, (hipStream_t)stream, dp);
    return (int)hipGetLastError();
}

int launch_derive(const DeriveParams &dp, void *stream)
{
    hipLaunchKernelGGL(derive_kernel, dim3((unsigned)dp.Hq), dim3(64), 0, (hipStream_t)stream, dp);
    hipLaunchKernelGGL(unify_schemes_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, dp.hp_table, dp.Hq, (uint32_t)dp.top);
    return (int)hipGetLastError();
}

} // namespace intattn
