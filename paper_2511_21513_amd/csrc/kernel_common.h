// Device helpers shared by the forward kernels: vector types, the exact index map of Sec. 3.1,
// the MFMA accumulator-to-key map and the LDS chunk swizzles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "params.h"

namespace intattn {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------------ workgroup -> work mapping
// Workgroups are dealt round-robin to the 8 XCDs (workgroup id mod 8), and each XCD has its
// own L2.  All query heads that share one KV head -- i.e. one (batch, KV head) group -- are
// therefore sent to the same XCD, so that K and V of the group are fetched into one L2 only.
// Within an XCD the groups are taken in batches of FwdParams::group_batch groups: inside a batch the longest
// (latest) causal query tiles of all its groups come first, which balances the compute units; the batch is sized
// so that the K and V its workgroups read at the same time fit the XCD's L2 (with the tiles of all 64 groups of
// an XCD interleaved, and no sharing between query heads, sweep C of the batched prefill workload streamed
// 4.3 TB/s of K and V from HBM and was bound by it).
constexpr int NUM_XCD = 8;
constexpr int64_t XCD_L2_BUDGET = 4 << 20; // bytes of K (and V) that a batch of groups may hold in flight: the L2 of an XCD
                                           // (1 to 16 MiB measured within 3 % of each other on the batched prefill workload)

// groups per batch for kernels that stream `bytes_per_group` of K (and V) per (batch, KV head) group
inline int fwd_group_batch(int B, int Hkv, int64_t bytes_per_group)
{
    const int64_t gpx = ((int64_t)B * Hkv + NUM_XCD - 1) / NUM_XCD;
    const int64_t fit = bytes_per_group > 0 ? XCD_L2_BUDGET / bytes_per_group : gpx;
    return (int)(fit < 1 ? 1 : (fit > gpx ? gpx : fit));
}

__host__ __device__ inline int64_t fwd_grid_size(int B, int Hq, int Hkv, int n_qtiles)
{
    const int64_t groups = (int64_t)B * Hkv;
    const int64_t groups_per_xcd = (groups + NUM_XCD - 1) / NUM_XCD;
    return (int64_t)NUM_XCD * groups_per_xcd * (Hq / Hkv) * n_qtiles;
}

struct WorkItem {
    int b, hq, kvh, qt;
    bool valid;
};

__device__ __forceinline__ WorkItem fwd_work_item(const FwdParams &p, int bid)
{
    const int g = p.group;
    const int groups = p.B * p.Hkv;
    const int groups_per_xcd = (groups + NUM_XCD - 1) / NUM_XCD;
    const int xcd = bid % NUM_XCD, slot = bid / NUM_XCD;
    const int gb = p.group_batch > 0 ? min(p.group_batch, groups_per_xcd) : groups_per_xcd;
    const int per_batch = g * gb * p.n_qtiles; // slots of a full batch; the last batch may hold fewer groups
    const int batch = slot / per_batch, rem = slot - batch * per_batch;
    const int gbb = min(gb, groups_per_xcd - batch * gb);
    const int hg = rem % g;
    const int j = batch * gb + (rem / g) % gbb;
    const int qt_rev = rem / (g * gbb);
    const int gi = j * NUM_XCD + xcd; // (batch, KV head) group
    WorkItem w;
    w.valid = gi < groups;
    w.b = gi / p.Hkv;
    w.kvh = gi % p.Hkv;
    w.hq = w.kvh * g + hg;
    w.qt = p.n_qtiles - 1 - qt_rev;
    return w;
}

// ------------------------------------------------------------------ index map (Sec. 3.1)
// The fp64 scheme's factor -r (its bits are split over idx_mul, low word, and idx_add).
__device__ __forceinline__ double idx_fp64_factor(const HeadParams &hp)
{
    return __builtin_bit_cast(double, ((uint64_t)hp.idx_add << 32) | (uint64_t)hp.idx_mul);
}

// t = -min(Delta, c_int) in [-c_int, 0]; returns round(-t * top / c_int).
template <int MODE>
__device__ __forceinline__ uint32_t index_map(int t, const HeadParams &hp, uint32_t top)
{
    if (MODE == IDX_MAD24) {
        // (-t) * mul + add, 24-bit signed operands (idx_mul holds -mul)
        return (uint32_t)(__mul24(t, (int)hp.idx_mul) + (int)hp.idx_add) >> hp.idx_shift;
    } else if (MODE == IDX_TOP24) {
        return (uint32_t)(__mul24(t, (int)hp.idx_mul) + (int)hp.idx_add) >> 24;
    } else if (MODE == IDX_MULHI24) {
        // high word of ((t << pre) - off) * (-mul): both factors negative 24-bit values
        const int x = (int)(((uint32_t)t << hp.idx_shift) + hp.idx_add); // idx_add holds -off
        int r;
        // written as an instruction so that later address arithmetic is not folded back into a
        // 64-bit product (which costs three more VALU operations per element)
        asm("v_mul_hi_i32_i24 %0, %1, %2" : "=v"(r) : "v"(x), "v"((int)hp.idx_mul));
        return (uint32_t)r;
    } else if (MODE == IDX_FP32) {
        // trunc(fma(t, -(top/c_int), 0.5)): t is exact in fp32, one rounding in the fma; the host
        // proved the result exact on the whole range with the same IEEE operations
        return (uint32_t)(int)__builtin_fmaf((float)t, __uint_as_float(hp.idx_mul), 0.5f);
    } else {
        // trunc(fma(t, -r, 0.5)) in IEEE fp64, r the double after top/c_int: exact for every c_int
        return (uint32_t)(int)__builtin_fma((double)t, idx_fp64_factor(hp), 0.5);
    }
}

// The map with the scheme named in the parameters themselves (pad[0]: chosen on the host, or by
// the derivation kernel for device-resident scales), for kernels where the map is not the hot loop.
__device__ __forceinline__ uint32_t index_any(const HeadParams &hp, int t, uint32_t top)
{
    switch (hp.pad[0]) {
    case IDX_MAD24: return index_map<IDX_MAD24>(t, hp, top);
    case IDX_TOP24: return index_map<IDX_TOP24>(t, hp, top);
    case IDX_MULHI24: return index_map<IDX_MULHI24>(t, hp, top);
    case IDX_FP32: return index_map<IDX_FP32>(t, hp, top);
    default: return index_map<IDX_FP64>(t, hp, top);
    }
}

// The same map applied to RAW scores of one query row (the lane's row): with the row maximum
// mx, idx = round(min(mx - s, c_int) * top / c_int).  The subtraction of mx is folded into
// per-row constants (all arithmetic is modulo 2^32 and the true values are small), so a
// score costs: clip (max with `bound`), then the scheme's two operations.
// Call with sc = max(s, bound), and additionally sc <= mx where hidden keys may exceed mx.
template <int MODE> struct RowIndex {
    int bound; // mx - c_int
    int mx;
    uint32_t addc;
    int mul;
    int shift;
    double negr; // fp64 schemes only (per lane when the parameters are per block of rows)

    __device__ __forceinline__ void init(const HeadParams &hp, int row_max, uint32_t top_)
    {
        mx = row_max;
        bound = row_max - hp.c_int;
        mul = (int)hp.idx_mul;
        shift = hp.idx_shift;
        negr = (MODE == IDX_FP64 || MODE == IDX_ROW64 || MODE == IDX_KGROUP) ? idx_fp64_factor(hp) : 0.0;
        (void)top_;
        if (MODE == IDX_MULHI24) addc = hp.idx_add - ((uint32_t)row_max << hp.idx_shift);
        else if (MODE == IDX_MAD24 || MODE == IDX_TOP24) addc = hp.idx_add - (uint32_t)__mul24(row_max, (int)hp.idx_mul);
        else addc = 0;
    }
    // Delta' * mul + add of the clipped score sc (IDX_TOP24: the index is its top byte)
    __device__ __forceinline__ uint32_t scaled(int sc) const { return (uint32_t)__mul24(sc, mul) + addc; }
    // Address of the score's entry in a table whose rows (one per index) are 256 bytes apart.  lane_base =
    // the table's address, which must be a multiple of 65536, plus the lane's offset (< 256) inside a
    // row.  IDX_TOP24: one byte permute puts the top byte of the scaled score into byte 1 of lane_base;
    // the other schemes shift the index up and add.
    __device__ __forceinline__ uint32_t row_addr(int sc, uint32_t lane_base) const
    {
        if (MODE == IDX_TOP24) return __builtin_amdgcn_perm(scaled(sc), lane_base, 0x03020700u);
        return ((*this)(sc) << 8) + lane_base;
    }
    __device__ __forceinline__ uint32_t operator()(int sc) const
    {
        if (MODE == IDX_MULHI24) {
            const int x = (int)(((uint32_t)sc << shift) + addc);
            int r;
            asm("v_mul_hi_i32_i24 %0, %1, %2" : "=v"(r) : "v"(x), "v"(mul));
            return (uint32_t)r;
        } else if (MODE == IDX_MAD24) {
            return ((uint32_t)__mul24(sc, mul) + addc) >> shift;
        } else if (MODE == IDX_TOP24) {
            return scaled(sc) >> 24;
        } else if (MODE == IDX_FP32) {
            return (uint32_t)(int)__builtin_fmaf((float)(sc - mx), __uint_as_float((uint32_t)mul), 0.5f);
        } else if (MODE == IDX_KGROUP) {
            // the fp64 map; the index is kept inside the table whatever an unusable scale produced
            return min((uint32_t)(int)__builtin_fma((double)(sc - mx), negr, 0.5), (uint32_t)shift); // shift holds 2^b - 1 here
        } else {
            return (uint32_t)(int)__builtin_fma((double)(sc - mx), negr, 0.5);
        }
    }
};

// The barrier that publishes tiles filled by direct-to-LDS loads: a wave's own loads must have landed before
// it signals, because the other waves read what it loaded.  (On this target the compiler also drains every
// counter before s_barrier; the wait is spelled out so that correctness does not rest on that.)
__device__ __forceinline__ void publish_tiles_barrier()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

// Key (within a 32-key block) held in accumulator register i of a 32x32 MFMA result by a
// lane of half-wave h; the same key sits in byte i of that lane's next B operand.
__device__ __forceinline__ int acc_key(int i, int h) { return 8 * (i >> 2) + 4 * h + (i & 3); }

// Eq. uint8-prob: round-half-up(255 E / S) = floor((510 E + S) / (2 S)) for E <= 255 and 1 <= S < 2^25, without an
// integer division: a single-precision estimate of the quotient (below 256, so off by one at most) corrected against
// the exact products.  inv_2s: the reciprocal of (float)(2 S) to within a few units in the last place (v_rcp_f32).
__device__ __forceinline__ uint32_t prob_u8(uint32_t e, uint32_t S, float inv_2s)
{
    const uint32_t num = 510u * e + S, den = 2u * S;
    uint32_t q = (uint32_t)((float)num * inv_2s);
    if (q * den > num) --q;
    if ((q + 1u) * den <= num) ++q;
    return q;
}

// Output requantization (Sec. 3.2): clamp(floor((acc * M + 2^(sh-1)) / 2^sh), -127, 127) with M < 2^31 and
// 1 <= sh <= 62.  For sh >= 33 (every ratio s_V / (255 s_O) below 1/4) the rounding addend lies wholly in the high
// word of the 64-bit product and the low word cannot change the floor of a division by 2^(sh-32) >= 2, so the
// high word alone gives the same value: multiply-high, add, shift.  FAST is the caller's statement that sh >= 33.
template <bool FAST> __device__ __forceinline__ int requant(int32_t acc, int32_t M, int32_t sh)
{
    int v;
    if (FAST) {
        v = (__mulhi(acc, M) + (1 << (sh - 33))) >> (sh - 32);
    } else {
        const int64_t w = ((int64_t)acc * M + (1ll << (sh - 1))) >> sh;
        v = w > 127 ? 127 : (w < -127 ? -127 : (int)w);
    }
    return v > 127 ? 127 : (v < -127 ? -127 : v);
}

// the same with the form chosen at run time (sh is uniform over a head)
__device__ __forceinline__ int requant_any(int32_t acc, int32_t M, int32_t sh)
{
    return sh >= 33 ? requant<true>(acc, M, sh) : requant<false>(acc, M, sh);
}

// XOR swizzles of the 16-byte chunk index inside a key row.
// K fragments are read with ds_read_b128, lane -> key row, all lanes of a half-wave on the same
// chunk.  The LDS serves 16 consecutive lanes (256 bytes, all 64 banks) per clock, so the 16 rows
// of such a group must land on 16 different 16-byte bank groups: rows 256 bytes apart share
// banks, and the swizzle separates exactly those (measured: 4.2 clocks per wave instruction
// against 7.6 with a swizzle that only separates 8 consecutive rows).
template <int D> __device__ __forceinline__ int swz_k(int key) { return D == 128 ? ((key >> 1) & 7) : ((key >> 2) & 3); }
template <int D> __device__ __forceinline__ int swz_v(int key)
{
    return D == 128 ? ((key & 3) | (((key >> 3) & 1) << 2)) : (((key >> 1) & 1) | (((key >> 3) & 1) << 1));
}

} // namespace intattn
