// Internal structures shared by the host side of the library and its kernels.
// Not part of the public ABI (that is include/intattn.h).
#pragma once
#include <stdint.h>

namespace intattn {

// How a kernel turns a clipped distance Delta' in [0, c_int] into the table index
// idx = round(Delta' * top / c_int)  (Sec. 3.1 index map), exactly.
enum IdxMode : int32_t {
    IDX_FP64 = 0,   // trunc(fma(Delta', r, 0.5)) in IEEE fp64, r = the double after top/c_int: exact for every c_int
                    // (idx_mul, idx_add hold the low and high word of the bits of -r)
    IDX_MAD24 = 1,  // (Delta' * mul + add) >> shift, 24-bit operands, 32-bit result
    IDX_MULHI24 = 2,// high 32 bits of the 48-bit product ((Delta' << pre) + add) * mul
    IDX_FP32 = 3,   // trunc(fma(Delta', top/c_int, 0.5)) in IEEE fp32 (idx_mul holds the bits of -top/c_int)
    IDX_DEVICE = 4, // launchers only: the scheme (TOP24 or FP64, one for all heads of the call) is in the HeadParams, written on the device
    IDX_ROW64 = 5,  // the fp64 scheme with parameters per block of query rows (FwdParams::row_table): finer
                    // quantization groups over the query rows, Sec. 3.3
    IDX_KGROUP = 7, // per-logit parameters: quantization groups over the key axis (Sec. 3.3), fp64 map per key block
    IDX_TOP24 = 6,  // MAD24 with shift 24: the index is the top byte of Delta' * mul + add, which one byte
                    // permute turns into the address of a table row 256 bytes apart (sweep C)
    IDX_MIX = 8     // launchers of sweep C only: every head's own scheme, IDX_TOP24 or IDX_MULHI24, is in its parameters
};

// Per query head: everything the kernel needs that depends on the scales.
struct HeadParams {
    int32_t c_int;     // clip threshold of Eq. clipping_thr, capped at 2^30
    uint32_t idx_mul;  // index-map multiplier (see IdxMode)
    uint32_t idx_add;  // index-map addend
    int32_t idx_shift; // MAD24: right shift; MULHI24: left pre-shift of Delta'
    int32_t rq_mult;   // output requantization multiplier M in [2^30, 2^31)
    int32_t rq_shift;  // output requantization shift sh in [1, 62]
    int32_t pad[2];    // pad[0]: this head's IdxMode when the table was derived on the device
};

struct FwdParams {
    const int8_t *q, *k, *v;
    int8_t *out;
    int64_t qs[3], ks[3], vs[3], os[3]; // byte strides of B, H, L
    int32_t B, Hq, Hkv;
    int32_t L;           // query rows
    int32_t Lk;          // keys
    int32_t row_lo;      // number of the first query row in the numbering where row r sees keys <= r under the
                         // causal mask: Lk - L when causal, else 0; tiles are aligned to this numbering
    int32_t causal;
    int32_t group;       // Hq / Hkv
    int32_t top;         // 2^b - 1
    int32_t n_qtiles;    // tiles of (rows per workgroup) rows that [row_lo, row_lo + L) touches
    int32_t n_chunks;    // ceil(Lk / rows per workgroup of sweep C): chunks of V the column sums are kept for
    const HeadParams *hp_table; // device [Hq] when per-head or derived on the device, else nullptr
    const HeadParams *hp_table_c; // device [Hq] or nullptr: sweep C's own table (IDX_MIX) where some heads have top-byte constants
    const HeadParams *row_table; // IDX_ROW64: device [B * Hq][n_rowblk], parameters of every block of q_block query rows
    int32_t q_block, n_rowblk;
    // IDX_KGROUP: scales per block of q_block query rows [B * Hq][n_rowblk] and per block of k_block keys
    // [B * Hkv][n_kblk] (device), the clip bound c and sqrt(d), and the per-head status words (non-zero: zeros out)
    const float *sq_rows, *sk_blocks;
    int32_t k_block, n_kblk;
    double clip, sqrt_d;
    const int32_t *head_status;
    int32_t filter;             // 1: a workgroup whose head's HeadParams name another scheme than the kernel's returns at once
    int32_t group_batch;        // (batch, KV head) groups of an XCD whose query tiles are interleaved; 0: all of them
    HeadParams hp0;             // the single parameter set when hp_table == nullptr
    uint32_t lut[16];           // LUT_hat, up to 64 bytes packed little-endian (unused tail is 0)
    int32_t *dbg_row_max, *dbg_row_sum, *dbg_acc;
    // workspace: [B*Hq*L] row max and [B*Hq*L] row sum (handed from the first to the second launch
    // of the two-launch variants), [B*Hkv*n_chunks*d] sums of V over each chunk of keys
    int32_t *ws_row_max, *ws_row_sum, *ws_colsum;
    // split-key path for few query rows (decode): packed rows (Hq / Hkv) * L, 32-key sub-tiles 4 * ceil(Lk / 128);
    // per (batch, KV head) group g and sub-tile j: raw scores [g][j][2][rows][16], table indices (16 bytes where the
    // scores have 16 words), partial row max and row sum [g][dec_np][rows]; partial accumulators per workgroup [g][dec_np / 4][rows][d]
    int32_t dec_rows, dec_nt32;
    int32_t dec_tpw, dec_np; // 128-key tiles per workgroup; partial maxima / sums per row = 4 * ceil(tiles / dec_tpw)
    int32_t *dec_scores, *dec_idx, *dec_pmax, *dec_psum, *dec_acc;
    // fused split-key kernel: DEC_STATE_WORDS words per (batch, KV head) group, zero between launches (arrival and
    // departure counters of the group's workgroups, row maxima, row sums); nullptr: the separate launches
    uint32_t *dec_state;
    int32_t dec_spin_limit; // polls of a group counter before a workgroup gives up (and raises the group's status word)
    int32_t dec_wide;       // 1: the fused kernel keeps raw 32-bit scores in LDS (any clip threshold; chunks half as long)
    // comparator only
    float alpha0, sv_over_so0;  // per-tensor values when the float tables are null
    const float *alpha_table;   // device [Hq]
    const float *svso_table;    // device [Hq]
};

constexpr int DEC_STATE_WORDS = 96; // [0] arrivals, [1] departures, [2] status, [32, 63) row maxima (biased), [64, 95) row sums

// Arguments of the dynamic quantizer (Sec. 2.1, Eq. quant).
struct QuantParams {
    const void *src;       // [B, H, L, d], d contiguous
    int8_t *dst;
    int64_t ss[3], ds[3];  // byte strides of B, H, L
    int32_t B, H, L, d;
    int32_t dtype;         // 0 fp32, 1 fp16, 2 bf16
    int32_t per_head;      // 0: one scale; 1: one per head index; 2: one per block of q_block rows of every (b, h)
    int32_t q_block;
    float *scales;         // device, 1 or H values (out)
    float *partial;        // device scratch: max|X| of every workgroup of the first pass, [B * H][n_partial]
    int32_t n_partial;
};

// Up to four tensors quantized by one pair of launches: workgroups [first[i], first[i + 1]) of the flat grid
// belong to tensor i; gx[i] = workgroups along the items of one (b, h) slice in the second pass.
struct QuantBatch {
    QuantParams t[4];
    int32_t n;
    uint32_t first[5];
    uint32_t gx[4];
};

// Arguments of IndexSoftmax as an operator on INT32 logits (Sec. 3.1-3.2).
struct SoftmaxParams {
    const int32_t *logits; // device [rows, cols]
    uint8_t *prob;         // device [rows, cols]
    int64_t ls, ps;        // byte strides of a row
    int64_t rows;
    int32_t cols;
    int32_t rows_per_matrix, causal; // causal: row r of each stacked matrix sees columns j <= r % rows_per_matrix + cols - rows_per_matrix
    int32_t top;           // 2^b - 1
    int32_t vec_in, vec_out; // rows start 16-byte (logits) / 4-byte (prob) aligned: wide loads / stores
    HeadParams hp;         // c_int and the index-map constants, scheme in pad[0]
    uint32_t lut[16];
};

// Arguments of the derivation of HeadParams from device-resident scales.
struct DeriveParams {
    const float *scale_q, *scale_k, *scale_v, *scale_out; // device; scale_out may be null (= scale_v)
    int32_t per_head;      // 0: one value each; 1: scale_q/out per query head, scale_k/v per KV head
    int32_t Hq, group, top;
    double clip, sqrt_d;
    HeadParams *hp_table;  // device [Hq] (out; all heads also when the scales are per tensor)
    int32_t *status;       // device [Hq] (out): 1 where a head's scales were unusable, else 0
    // per block of query rows (launch_derive_rows): scale_q / scale_out hold n_entries = B * Hq * n_rowblk values
    int64_t n_entries;
    int32_t n_rowblk;
    HeadParams *row_table; // device [n_entries] (out)
    // groups over the key axis as well (launch_derive_groups): scale_k holds n_kentries = B * Hkv * n_kblk values,
    // one per block of keys; the row table then carries the requantization of each block of query rows only
    int64_t n_kentries;
    int32_t n_kblk, Hkv;
};

// Launchers implemented in the .hip files.  Return a hipError_t cast to int.
// stage 0: everything; 1: V column sums + sweeps A+B; 2: sweep C (two-launch variants only; else hipErrorNotSupported)
int launch_fwd(const FwdParams &p, int d, int idx_mode, int variant, int stage, void *stream);
int launch_sweep_c(const FwdParams &p, int d, int idx_mode, void *stream);
int launch_fwd_splitk(const FwdParams &p, int d, int idx_mode, void *stream);
int fwd_choose_variant(int variant, int B, int Hq, int L, int Lk, int d, int causal); // resolves 0 (automatic) to a concrete variant
int fwd_rows_per_block(int variant);
// tiles of `rows_per_tile` rows, aligned to multiples of it, that rows [row_lo, row_lo + n_rows) touch
inline int fwd_row_tiles(int row_lo, int n_rows, int rows_per_tile)
{
    return (row_lo + n_rows + rows_per_tile - 1) / rows_per_tile - row_lo / rows_per_tile;
}
bool fwd_variant_known(int variant);
int quantize_partials_per_slice(int B, int H, int L, int d);
int launch_quantize(const QuantParams *ps, int n, void *stream);
int launch_decode(const FwdParams &p, int d, void *stream);
int launch_index_softmax(const SoftmaxParams &p, void *stream);
int launch_derive(const DeriveParams &dp, void *stream);
int launch_derive_rows(const DeriveParams &dp, void *stream);
int launch_derive_groups(const DeriveParams &dp, void *stream);
int launch_quantonly(const FwdParams &p, int d, int variant, void *stream);

} // namespace intattn
