/*
 * intattn.h -- C ABI of the MI355X (gfx950) fused integer attention library.
 *
 * The library computes the IntAttention pipeline of arxiv 2511.21513 in one fused
 * pass per (batch, head, query tile), entirely in integers:
 *
 *   A_hat  = Q_hat . K_hat^T            INT8 x INT8 -> INT32   (Sec. 2.1, Eq. logit-scale)
 *   Delta  = rowMax(A_hat) - A_hat      (Sec. 3.1)
 *   Delta' = min(Delta, c_int),  c_int = round(c * sqrt(d) / (s_Q * s_K))
 *                                       (Sec. 3.1, Eq. clipping_thr, Eq. int_clipping)
 *   idx    = round(Delta' * (2^b - 1) / c_int)                  (Sec. 3.1, index map)
 *   E_hat  = LUT_hat[idx],  LUT_hat[i] = round(255 * exp(-c*i/(2^b-1))), last entry 0
 *                                       (Sec. 3.1 Eq. lut_re, Sec. 3.2 Eq. lut16, Eq. gather16)
 *   P_hat  = round(255 * E_hat / rowSum(E_hat))    UINT8        (Sec. 3.2, Eq. uint8-prob)
 *   acc    = P_hat . V_hat              UINT8 x INT8 -> INT32   (Sec. 2.1 Eq. pv-link, Sec. 3)
 *   out    = clamp(round(acc * s_V / (255 * s_O)), -127, 127)   INT8
 *
 * "round" is round-half-up; for idx, P_hat and out it is evaluated in exact integer
 * arithmetic.  The output requantization is a fixed-point multiply-shift: with
 * r = s_V / (255 s_O) = m * 2^e, m in [0.5, 1), M = round(m * 2^31), sh = 31 - e,
 * out = clamp(floor((acc * M + 2^(sh-1)) / 2^sh), -127, 127).  The paper states no
 * requantization formula; this one follows from Eq. pv-link with P = P_hat / 255.
 * With causal != 0, key j is visible to query i iff j <= i (j <= i + Lkv - L when the
 * key sequence is longer than the query block); hidden keys take no part in rowMax /
 * rowSum and get P_hat = 0.  Query head h reads KV head h / (Hq / Hkv).
 * Per-head scales are the group-wise form of Sec. 3.3 with one group per head; scale
 * mode 2 has one group per block of query rows (per token at block size 1).
 *
 * Around that path: intattn_quantize (Sec. 2.1, Eq. quant, scales left in device memory),
 * intattn_forward_dynamic (the forward on such device-resident scales) and
 * intattn_index_softmax (Sec. 3.1-3.2 alone, on INT32 logits).
 *
 * The L x L score matrix never reaches HBM.  Results are a deterministic integer
 * function of the inputs (no dependence on tiling or launch shape).
 *
 * All entry points return 0 on success or a negative INTATTN_ERR_* code; none throws or aborts.
 * A forward call enqueues its kernels and returns; it allocates device memory (hipMalloc / hipFree,
 * which wait for the device) only when the problem needs a larger workspace or table than any call
 * before it on this context did -- intattn_reserve does that ahead of time, and
 * intattn_forward_noalloc never allocates.  Small per-head tables reach the device through pinned
 * staging buffers of the context (two of them; a third upload while two are still in flight waits
 * for the oldest).  intattn_dynamic_status reads a word back and so waits for its copy.
 * A context is bound to one device and is not thread-safe; calls that share a context must be
 * issued on one stream at a time.
 */
#ifndef INTATTN_H
#define INTATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define INTATTN_API __attribute__((visibility("default")))

#define INTATTN_OK 0
#define INTATTN_ERR_INVALID_ARG (-1) /* null / negative / misaligned / inconsistent argument */
#define INTATTN_ERR_UNSUPPORTED (-2) /* valid request outside what the kernels cover          */
#define INTATTN_ERR_HIP (-3)         /* a HIP runtime call failed; see intattn_last_error     */
#define INTATTN_ERR_NOMEM (-4)       /* host or device allocation failed                      */

typedef struct intattn_ctx intattn_ctx; /* opaque; owned by the library */

typedef struct {
    int32_t device;   /* HIP device ordinal the context is bound to; -1 = host-only context
                         (parameter derivation and LUT only; forward calls are rejected)     */
    int32_t lut_bits; /* b of Sec. 3.1: the table has 2^b entries; 1..6; paper default 5     */
    double clip;      /* c of Sec. 3.1: clip threshold in logit units; > 0; paper default 6.6 */
    int32_t variant;  /* kernel variant: 0 = automatic choice.  Tuning knobs, all bit-identical: 1, 2 = one
                         launch with 32 / 64 query rows per wave; 3 = one launch, a workgroup per 32 query
                         rows with the keys split over its waves (small and mid-size problems); 4, 5 = two
                         launches (row max and row sum, then P.V) with the phase-ordered / the
                         software-pipelined second kernel;
                         9 = the split-key path for few query rows wherever the shape allows (one launch
                         whose workgroups meet at counters in device memory; intattn_forward_noalloc
                         takes four launches);
                         10 = the split-key path with the four launches always.
                         Other values are rejected                                                    */
    int32_t reserved; /* must be 0                                                           */
} intattn_config;

/*
 * One forward call.  Tensors are logically [B, H, L, d] with d contiguous; the three
 * strides per tensor are ELEMENT (= byte) strides of the B, H and L axes.  Every tensor
 * pointer and every stride must be a multiple of 16.  out must not alias the inputs.
 * Device buffers are borrowed until the stream reaches the end of the enqueued work;
 * host scale arrays are read before the call returns.
 */
typedef struct {
    int32_t B, Hq, Hkv, L, d; /* Hq % Hkv == 0; d in {64, 128}; 1 <= L <= 131071 query rows   */
    int32_t causal;           /* 0 or 1                                                       */
    const int8_t *q;          /* DEVICE  [B, Hq,  L, d]                                       */
    const int8_t *k;          /* DEVICE  [B, Hkv, Lkv, d]                                     */
    const int8_t *v;          /* DEVICE  [B, Hkv, Lkv, d]                                     */
    int8_t *out;              /* DEVICE  [B, Hq,  L, d]                                       */
    int64_t q_stride[3], k_stride[3], v_stride[3], out_stride[3];
    int32_t scale_mode;       /* 0: one float per scale array; 1: per head ([Hq] for q and
                                 out, [Hkv] for k and v), shared over the batch; 2
                                 (intattn_forward_dynamic only): finer groups over the query
                                 rows, Sec. 3.3 -- scale_q and scale_out hold one value per
                                 block of q_block consecutive query rows of every (batch,
                                 head), [B, Hq, ceil(L / q_block)] (q_block = 1: per token);
                                 scale_k and scale_v one per KV head; 3 (intattn_forward_dynamic
                                 only): groups over both axes, Sec. 3.3 -- scale_q / scale_out
                                 as in mode 2, scale_k one value per block of k_block
                                 consecutive keys of every (batch, KV head),
                                 [B, Hkv, ceil(Lkv / k_block)] (k_block = 1: per key, i.e. per
                                 output channel of Q.K^T; multiples of 32 run fastest),
                                 scale_v one per KV head.  The row maximum is taken over the
                                 dequantized logits alpha^(g) A_hat in fp64 and every key
                                 block measures distances from round(M / alpha^(g)) with its
                                 own c_int^(g) (capped at 2^30); one row sum over all keys.
                                 dbg_row_max is not written in this mode                      */
    int32_t Lkv;              /* number of keys / values; 0 means L (square self-attention).
                                 Lkv != L: a chunk of queries, or one decoded token, against a
                                 longer (or, without mask, any) key sequence; the causal mask
                                 is then aligned to the end, key j visible to query i iff
                                 j <= i + Lkv - L, and needs Lkv >= L                         */
    const float *scale_q;     /* HOST */
    const float *scale_k;     /* HOST */
    const float *scale_v;     /* HOST */
    const float *scale_out;   /* HOST, or NULL: s_O = s_V of the matching KV head             */
    int32_t *dbg_row_max;     /* optional DEVICE [B, Hq, L] contiguous: rowMax(A_hat); NULL off */
    int32_t *dbg_row_sum;     /* optional DEVICE [B, Hq, L] contiguous: rowSum(E_hat); NULL off */
    int32_t *dbg_acc;         /* optional DEVICE [B, Hq, L, d] contiguous: P_hat.V_hat; NULL off */
    int32_t q_block;          /* scale_mode 2 only: query rows per quantization group, >= 1   */
    int32_t k_block;          /* scale_mode 3 only: keys per quantization group, >= 1; else 0 */
} intattn_args;

/* Builds LUT_hat for (lut_bits, clip) (Sec. 3.1 Eq. lut_re, Sec. 3.2 Eq. lut16) and binds the
 * context to cfg->device.  *out receives the context; release it with intattn_destroy. */
INTATTN_API int intattn_create(intattn_ctx **out, const intattn_config *cfg);

/* Enqueues the fused IntAttention forward (Sec. 3) on hip_stream (a hipStream_t; NULL is
 * the default stream) and returns without waiting for it.  The context owns a device workspace
 * (8 bytes per query row plus d int32 per 128 keys and KV head) that the first call allocates and
 * a later, larger call re-allocates (hipMalloc / hipFree wait for the device and are not for use
 * under graph capture: call intattn_reserve first, or use intattn_forward_noalloc); the
 * kernels of a call pass intermediate results through it, so calls on ONE context must not
 * overlap in time (same stream, or ordered by the caller); use one context per concurrent stream.
 * The one-launch split-key path (few query rows; see intattn_config.variant) lets the workgroups of a
 * (batch, KV head) group wait for each other at a counter in device memory.  Alone on the GPU a group's
 * workgroups are always scheduled together (they have consecutive ids).  The wait is bounded (a few
 * seconds): where other work keeps a group from being scheduled together for that long -- another process
 * that fills the GPU, or two calls of this path running at the same time on different streams, each
 * holding compute units the other's groups wait for -- the workgroups give up, the call's output is
 * undefined and so are later calls of this path on the context until intattn_reserve has cleared the
 * counters.  Order such calls on one stream, or use variant 10, which never waits.  (Testing aid: the
 * environment variable INTATTN_SPLITKEY_SPIN_LIMIT, read at every such call, lowers the bound, counted in
 * polls of the counter.) */
INTATTN_API int intattn_forward(intattn_ctx *ctx, const intattn_args *args, void *hip_stream);

/* Pre-sizes the context's device memory (workspace, per-head tables) for a problem of the shape and
 * scale mode of `args`, so that later forward calls with problems no larger allocate nothing and
 * never wait for the device.  dynamic != 0: for intattn_forward_dynamic (scale pointers are not read
 * either way).  May call hipMalloc / hipFree; launches nothing. */
INTATTN_API int intattn_reserve(intattn_ctx *ctx, const intattn_args *args, int32_t dynamic);

/* intattn_forward for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments (host scales), same kernels, same
 * bytes out, but the workspace -- row maxima and row sums between the launches, V column sums, the
 * partial results of the split-key kernels -- and the per-head parameter table live in a static
 * device array of INTATTN_NOALLOC_SCRATCH_BYTES that the library's image holds on every GPU it runs
 * on.  Calls no hipMalloc / hipFree.  A problem that needs more workspace than the array holds (8
 * bytes per query row of every (batch, head) plus 4 d bytes per 128 keys of every (batch, KV head),
 * or more than 512 query heads with per-head scales) is rejected with INTATTN_ERR_UNSUPPORTED and a
 * message naming both sizes.  The array is shared by every context on the GPU and keeps the last
 * call's contents (everything a call reads it has written first): calls that overlap in time on one
 * GPU race -- order them on one stream.
 * Under graph capture: with per-tensor scales (scale_mode 0) the call records kernels only.  With per-head
 * scales it also copies the parameter table from a host staging buffer of the context on every call, and a
 * replayed graph would copy whatever that buffer holds by then: capture intattn_forward instead (after one
 * eager call with the same scales the table is resident and the captured call records kernels only), or
 * intattn_forward_dynamic, which derives the parameters on the device. */
#define INTATTN_NOALLOC_SCRATCH_BYTES (4u << 20)
INTATTN_API int intattn_forward_noalloc(intattn_ctx *ctx, const intattn_args *args, void *hip_stream);

/* Timing hook for benchmarks, not part of the serving interface: the forward cut at the point where
 * the row maxima and row sums of IndexSoftmax (Sec. 3.1-3.2) are complete, so that the two launches of
 * the tiled path can be timed separately.  stage 0: everything, as
 * intattn_forward.  stage 1: V column sums and sweeps A+B only (row max, row sum of E_hat go to
 * the context's workspace; args->out is not written).  stage 2: sweep C only (P_hat, P_hat.V_hat,
 * requantization), reading what the last stage-1 call on this context left: it must have had the
 * same arguments, and nothing else may run on the context in between.  Returns
 * INTATTN_ERR_UNSUPPORTED when the kernel variant in use for this problem is a single launch. */
INTATTN_API int intattn_forward_stage(intattn_ctx *ctx, const intattn_args *args, void *hip_stream, int32_t stage);

/* intattn_forward for scales that live in DEVICE memory, e.g. where intattn_quantize left them
 * (Sec. 2.1 dynamic quantization feeding Sec. 3): args->scale_q / scale_k / scale_v / scale_out
 * are DEVICE pointers here (same counts as for intattn_forward; scale_out may be NULL), every
 * other field is as there.  scale_mode 2 (one scale per block of q_block query rows, Sec. 3.3) is
 * served by this entry only.  A small kernel on hip_stream derives each head's c_int (Sec. 3.1,
 * Eq. clipping_thr), requantization multiplier and index-map constants from them with the host
 * path's arithmetic, so the output is bit-identical to intattn_forward with the same scale
 * values, and the host never reads the scales: quantizer and attention can be enqueued back to
 * back.  Scales that are not finite and > 0 (or a ratio s_V / (255 s_O) outside the multiplier's
 * range) cannot be reported by return code: the affected heads' output is then all zeros, and
 * intattn_dynamic_status reports it.  Same workspace and no-overlap rules as intattn_forward. */
INTATTN_API int intattn_forward_dynamic(intattn_ctx *ctx, const intattn_args *args, void *hip_stream);

/* *status (HOST) = 1 if the last intattn_forward_dynamic on this context met an unusable scale,
 * else 0.  Copies one word from the device with a blocking copy; call it after synchronizing the
 * stream that call was enqueued on. */
INTATTN_API int intattn_dynamic_status(intattn_ctx *ctx, int32_t *status);

/*
 * IndexSoftmax as an operator of its own (Sec. 3.1-3.2; the paper's softmax-only setting): INT32
 * logits in, UINT8 probabilities out, per row
 *   P = round(255 * LUT_hat[round(min(rowMax - A, c_int) * (2^b - 1) / c_int)] / rowSum(LUT_hat[...])).
 * The table is the context's (lut_bits, clip); c_int comes from the caller (intattn_derive_params
 * computes it from scales, Eq. clipping_thr).
 */
typedef struct {
    int64_t rows;            /* >= 1                                                          */
    int32_t cols;            /* 1 .. 2^29                                                     */
    int32_t c_int;           /* clip threshold in logit units, 1 .. 2^30                      */
    const int32_t *logits;   /* DEVICE [rows, cols]                                           */
    uint8_t *prob;           /* DEVICE [rows, cols]; must not alias logits                    */
    int64_t logits_stride;   /* BYTES between rows, >= 4 * cols, multiple of 4                */
    int64_t prob_stride;     /* BYTES between rows, >= cols.  Rows that all start 16-byte
                                (logits) and 4-byte (prob) aligned take the wide accesses     */
    int32_t causal;          /* 0, or 1: the rows are stacked [rows_per_matrix, cols] matrices
                                with the attention mask: row r of a matrix sees columns
                                j <= r + cols - rows_per_matrix; hidden columns get 0          */
    int32_t rows_per_matrix; /* used when causal: >= 1, <= cols, divides rows                 */
} intattn_softmax_args;

/* Enqueues the operator on hip_stream and returns without waiting.  Allocates nothing. */
INTATTN_API int intattn_index_softmax(intattn_ctx *ctx, const intattn_softmax_args *args, void *hip_stream);

/* In-run comparator: the conventional INT8 pipeline the paper calls "Quant-Only"
 * (Sec. 2.2): INT8 Q.K^T, dequantize to fp32 with alpha, fp32 softmax, requantize P to
 * signed INT8 (x127), INT8 P.V, requantize the output with the same s_O.  Same arguments
 * and launch shape as intattn_forward; results are close to, not equal to, fp softmax
 * attention.  dbg_* taps are ignored. */
INTATTN_API int intattn_forward_quantonly(intattn_ctx *ctx, const intattn_args *args, void *hip_stream);

/* Arguments of intattn_quantize.  src and dst are DEVICE pointers to [B, H, L, d] tensors with byte
 * strides for B, H, L (d contiguous, d a multiple of 8; src and its strides multiples of 16
 * bytes, dst and its strides multiples of 8); scales is a DEVICE array of 1 (scale_mode 0), H (scale_mode 1) or
 * B * H * ceil(L / q_block) (scale_mode 2) floats that receives the scales.  The caller owns all three. */
typedef struct intattn_quant_args {
    int32_t B, H, L, d;
    int32_t dtype;       /* element type of src: 0 = fp32, 1 = fp16, 2 = bf16 */
    int32_t scale_mode;  /* 0 = one scale for the tensor, 1 = one per head index (shared over the batch),
                            2 = one per block of q_block consecutive rows of every (b, h) slice
                            (Sec. 3.3; q_block = 1: per token): scales is [B, H, ceil(L / q_block)] */
    const void *src;
    int8_t *dst;
    int64_t src_stride[3];
    int64_t dst_stride[3];
    float *scales;
    int32_t q_block;     /* scale_mode 2 only: rows per group, >= 1 */
    int32_t reserved;    /* must be 0 */
} intattn_quant_args;

/* Dynamic symmetric INT8 quantization of one of Q, K, V (Sec. 2.1, Eq. quant): s = max|X| / 127
 * over the tensor (or over each head index), X_hat = clamp(round(X / s), -127, 127), computed in
 * fp32 (the result of one IEEE division per element, ties to even; max|X| is floored at 1e-12).  Enqueued on
 * hip_stream; the scales stay in device memory.  Inputs must be finite.  Uses a small scratch
 * buffer of the context (allocated by the first call, B * H <= 65535). */
INTATTN_API int intattn_quantize(intattn_ctx *ctx, const intattn_quant_args *args, void *hip_stream);

/* intattn_quantize for `count` tensors at once (1..4; typically Q, K and V of one layer, Sec. 2.1,
 * Eq. quant): args points at `count` consecutive argument structs, each as for intattn_quantize with
 * scale_mode 0 or 1 (shapes, element types and scale modes may differ; a tensor with scale_mode 2
 * goes alone).  Same results as separate calls, in two kernel launches for the whole batch instead of
 * two per tensor.  Same scratch buffer and ordering rules. */
INTATTN_API int intattn_quantize_batch(intattn_ctx *ctx, const intattn_quant_args *args, int32_t count, void *hip_stream);

/* Host-only parameter derivation, exposed for tests: c_int of Eq. clipping_thr for
 * (s_q, s_k, d), and the output multiplier/shift for (s_v, s_o).  Any output pointer may be
 * NULL.  Returns INTATTN_ERR_INVALID_ARG for non-positive scales or an unrepresentable ratio. */
INTATTN_API int intattn_derive_params(const intattn_ctx *ctx, float s_q, float s_k, float s_v, float s_o,
                          int32_t d, int64_t *c_int, int32_t *rq_mult, int32_t *rq_shift);

/* Host-only, exposed for tests: how the kernels evaluate the index map of Sec. 3.1,
 * idx = round(x * (2^b - 1) / c_int) for x in [0, c_int], without dividing.  On entry *mode
 * names the scheme asked for; on return it is that scheme, or 0 if no constants exist for it
 * (the kernels then use scheme 0, which exists for every c_int).  Every scheme is checked
 * against the exact quotient at both sides of every index step before it is returned.
 *   mode 0: idx = trunc(fma(x, r, 0.5)) in IEEE fp64, *mul / *add = low / high word of the bits of r
 *   mode 1: idx = (x * mul + add) >> shift                 (32-bit sum, 24-bit factors)
 *   mode 2: idx = (((x << shift) + add) * mul) >> 32       (48-bit product of 24-bit factors)
 *   mode 3: idx = trunc(fma(x, r, 0.5)) in IEEE fp32, *mul = the bits of r; add = shift = 0
 *   mode 6: mode 1 with shift = 24: the index is the top byte of x * mul + add */
INTATTN_API int intattn_derive_index_map(const intattn_ctx *ctx, int64_t c_int, int32_t *mode, uint32_t *mul,
                                         uint32_t *add, int32_t *shift);

/* Copies the 2^b bytes of LUT_hat to dst (HOST); cap is dst's capacity in bytes.
 * Returns the number of bytes written, or a negative error. */
INTATTN_API int intattn_get_lut(const intattn_ctx *ctx, uint8_t *dst, int32_t cap);

/* Text of the last error recorded on ctx (never NULL; empty if none).  With ctx == NULL,
 * the text of the last failed intattn_create on this thread. */
INTATTN_API const char *intattn_last_error(const intattn_ctx *ctx);

/* Releases the context and the device memory it owns.  NULL is allowed. */
INTATTN_API void intattn_destroy(intattn_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* INTATTN_H */
