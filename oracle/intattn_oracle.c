/*
 * intattn_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded CPU statement of what the IntAttention
 * pipeline computes: INT8 Q.K^T -> IndexSoftmax -> UINT8 P times INT8 V ->
 * INT8 output.  Every step is written in the order and notation of the paper
 * (Sec. 2.1 "Attention and Dynamic Quantization", Sec. 3.1 "IndexSoftmax",
 * Sec. 3.2 "LUT Rebuild and Integer Scale Normalization", Sec. 3.3
 * "Quantization Scope and Compatibility").  All integer work is done in
 * int64_t, one query row at a time, with no blocking, fusion or reordering.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use
 * this file.  It shares no code, header, table or constant with the HIP
 * library; the HIP library never calls it.
 *
 * Readings taken where the paper is silent (each is also what the HIP path
 * implements, and each is listed in the design notes):
 *   - "round" (the floor-ceil bracket of Eq. clipping_thr, the index map,
 *     Eq. lut16, Eq. uint8-prob) is round-half-up.  For the index map and
 *     Eq. uint8-prob it is evaluated in exact integer arithmetic:
 *     round(x/y) = floor((2x + y) / (2y)) for y > 0.
 *   - Eq. quant (the dynamic quantizer in front of the path) works on fp32
 *     values: the scale is one fp32 division, every element one fp32 division
 *     rounded to the nearest integer with ties to even (the default IEEE
 *     rounding of rintf); max|X| is floored at 1e-12 so that an all-zero group
 *     has a scale.
 *   - causal masking: key j is visible to query i iff j <= i; hidden keys take
 *     no part in rowMax or rowSum and get P = 0.
 *   - rectangular shapes (L query rows against Lk != L keys; the paper states
 *     the square case only): every row is processed as before over its visible
 *     keys; a causal mask is aligned to the end, key j visible to query i iff
 *     j <= i + (Lk - L), which needs Lk >= L.  Pinned to the square problem (the
 *     last L rows of the Lk x Lk problem are these rows).
 *   - grouped-query attention: query head h reads KV head h / (Hq/Hkv).
 *   - the output is requantized with a fixed-point multiplier (M, sh) that
 *     encodes r = s_V / (255 * s_O)  (Eq. pv-link with P = P_hat/255):
 *     out = clamp(floor((acc*M + 2^(sh-1)) / 2^sh), -127, 127).
 *     PARITY UNPINNED by the paper: the paper prints no requantization formula.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_NO_MEM (-2)

/* floor(a / b) for b > 0, any sign of a (C's '/' truncates toward zero). */
static int64_t floor_div(int64_t a, int64_t b)
{
    int64_t q = a / b;
    int64_t r = a % b;
    if (r != 0 && r < 0) q -= 1;
    return q;
}

/* round-half-up of the rational x / y, y > 0, x >= 0 or x < 0. */
static int64_t round_div(int64_t x, int64_t y)
{
    return floor_div(2 * x + y, 2 * y);
}

/*
 * Eq. lut_re followed by Eq. lut16:
 *   LUT[i]     = exp(-c * i / (2^b - 1))   for 0 <= i < 2^b - 1,   LUT[2^b - 1] = 0
 *   LUT_hat[i] = round(255 * LUT[i])
 * lut must hold 2^b bytes.  1 <= b <= 8.
 */
int intattn_oracle_lut(int lut_bits, double clip, uint8_t *lut)
{
    if (lut_bits < 1 || lut_bits > 8 || !(clip > 0.0) || lut == NULL) return ORACLE_BAD_ARG;
    int n = 1 << lut_bits;
    for (int i = 0; i < n - 1; ++i) {
        double e = exp(-clip * (double)i / (double)(n - 1));
        lut[i] = (uint8_t)floor(255.0 * e + 0.5);
    }
    lut[n - 1] = 0;
    return ORACLE_OK;
}

/*
 * Eq. logit-scale and Eq. clipping_thr:
 *   alpha = s_Q * s_K / sqrt(d),   c_int = round(c / alpha).
 * A threshold below 1 is raised to 1 so that the index map never divides by 0.
 */
int64_t intattn_oracle_c_int(double clip, float s_q, float s_k, int d)
{
    double alpha = ((double)s_q * (double)s_k) / sqrt((double)d);
    double c = floor(clip / alpha + 0.5);
    if (!(c >= 1.0)) return 1;
    if (c > 4.0e18) return (int64_t)4000000000000000000LL;
    return (int64_t)c;
}

/*
 * Output requantization multiplier (reading; the paper gives only Eq. pv-link,
 * O ~= s_V * P * V_hat, and P_hat = 255 * P from Eq. uint8-prob).
 *   r = s_V / (255 * s_O) = m * 2^e with m in [0.5, 1);  M = round(m * 2^31);  sh = 31 - e.
 * Returns ORACLE_BAD_ARG when sh falls outside [1, 62].
 */
int intattn_oracle_requant_params(float s_v, float s_o, int64_t *mult, int32_t *shift)
{
    if (!(s_v > 0.0f) || !(s_o > 0.0f)) return ORACLE_BAD_ARG;
    double r = (double)s_v / (255.0 * (double)s_o);
    int e = 0;
    double m = frexp(r, &e);
    int64_t M = (int64_t)llround(m * 2147483648.0);
    if (M == 2147483648LL) { M = 1073741824LL; e += 1; }
    int sh = 31 - e;
    if (sh < 1 || sh > 62) return ORACLE_BAD_ARG;
    *mult = M;
    *shift = sh;
    return ORACLE_OK;
}

/* The index map of Sec. 3.1: idx = round(delta' * (2^b - 1) / c_int), exact. */
int64_t intattn_oracle_index(int64_t delta_clipped, int64_t c_int, int lut_bits)
{
    int64_t top = ((int64_t)1 << lut_bits) - 1;
    return round_div(delta_clipped * top, c_int);
}

/* Eq. uint8-prob for one element: round(255 * E / S), exact. */
int64_t intattn_oracle_prob(int64_t e, int64_t row_sum)
{
    return round_div(255 * e, row_sum);
}

typedef struct {
    int L, Lk, d, causal, lut_bits; /* L query rows, Lk keys */
    const int8_t *q;   /* [L, d] of this query head  */
    const int8_t *k;   /* [Lk, d] of the KV head     */
    const int8_t *v;   /* [Lk, d] of the KV head     */
    const uint8_t *lut;
    int64_t c_int;
    int64_t rq_mult;
    int32_t rq_shift;
    /* scratch, length Lk each */
    int64_t *a;
    int64_t *e;
    int64_t *p;
} head_ctx;

/* One query row i of one head, steps in the paper's order. */
static void oracle_row(const head_ctx *h, int i, int8_t *out /* [d] */, int32_t *row_max,
                       int32_t *row_sum, int32_t *acc_out /* [d] or NULL */,
                       uint8_t *prob_out /* [L] or NULL */)
{
    const int L = h->Lk, d = h->d;
    /* visible keys are 0 .. n_vis-1; with Lk != L the causal mask is aligned to the end (the last
     * query row sees every key): row i sees keys j <= i + (Lk - L) */
    const int n_vis = h->causal ? (i + (h->Lk - h->L) + 1) : L;

    /* Eq. logit-scale: A_hat[i, j] = sum_k Q_hat[i, k] * K_hat[j, k] */
    for (int j = 0; j < n_vis; ++j) {
        int64_t s = 0;
        for (int c = 0; c < d; ++c) s += (int64_t)h->q[(size_t)i * d + c] * (int64_t)h->k[(size_t)j * d + c];
        h->a[j] = s;
    }
    /* rowMax */
    int64_t m = h->a[0];
    for (int j = 1; j < n_vis; ++j)
        if (h->a[j] > m) m = h->a[j];

    /* Delta = m - A, Eq. int_clipping, index map, Eq. gather16, rowSum */
    int64_t S = 0;
    for (int j = 0; j < n_vis; ++j) {
        int64_t delta = m - h->a[j];
        int64_t dclip = delta < h->c_int ? delta : h->c_int;
        int64_t idx = intattn_oracle_index(dclip, h->c_int, h->lut_bits);
        h->e[j] = (int64_t)h->lut[idx];
        S += h->e[j];
    }
    /* Eq. uint8-prob */
    for (int j = 0; j < n_vis; ++j) h->p[j] = intattn_oracle_prob(h->e[j], S);

    if (prob_out) {
        for (int j = 0; j < L; ++j) prob_out[j] = (j < n_vis) ? (uint8_t)h->p[j] : 0;
    }
    if (row_max) *row_max = (int32_t)m;
    if (row_sum) *row_sum = (int32_t)S;

    /* P_hat * V_hat with integer accumulation, then requantization */
    const int64_t half = (int64_t)1 << (h->rq_shift - 1);
    const int64_t den = (int64_t)1 << h->rq_shift;
    for (int c = 0; c < d; ++c) {
        int64_t acc = 0;
        for (int j = 0; j < n_vis; ++j) acc += h->p[j] * (int64_t)h->v[(size_t)j * d + c];
        if (acc_out) acc_out[c] = (int32_t)acc;
        int64_t o = floor_div(acc * h->rq_mult + half, den);
        if (o > 127) o = 127;
        if (o < -127) o = -127;
        out[c] = (int8_t)o;
    }
}

static int check_problem(int B, int Hq, int Hkv, int L, int Lk, int causal, int d, int lut_bits, double clip,
                         const void *q, const void *k, const void *v, const float *sq,
                         const float *sk, const float *sv)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || L < 1 || Lk < 1 || d < 1) return ORACLE_BAD_ARG;
    if (causal && Lk < L) return ORACLE_BAD_ARG; /* a row without a visible key has no softmax */
    if (Hq % Hkv != 0) return ORACLE_BAD_ARG;
    if (lut_bits < 1 || lut_bits > 8 || !(clip > 0.0)) return ORACLE_BAD_ARG;
    if (!q || !k || !v || !sq || !sk || !sv) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

static int head_setup(head_ctx *hc, int Hq, int Hkv, int L, int Lk, int d, int causal, int b, int hq,
                      const int8_t *q, const int8_t *k, const int8_t *v, int scale_mode,
                      const float *sq, const float *sk, const float *sv, const float *so,
                      int lut_bits, double clip, const uint8_t *lut)
{
    const int g = Hq / Hkv;
    const int kv = hq / g;
    const float s_q = scale_mode ? sq[hq] : sq[0];
    const float s_k = scale_mode ? sk[kv] : sk[0];
    const float s_v = scale_mode ? sv[kv] : sv[0];
    const float s_o = so ? (scale_mode ? so[hq] : so[0]) : s_v;
    if (!(s_q > 0.0f) || !(s_k > 0.0f)) return ORACLE_BAD_ARG;
    hc->L = L;
    hc->Lk = Lk;
    hc->d = d;
    hc->causal = causal;
    hc->lut_bits = lut_bits;
    hc->q = q + ((size_t)b * Hq + hq) * (size_t)L * d;
    hc->k = k + ((size_t)b * Hkv + kv) * (size_t)Lk * d;
    hc->v = v + ((size_t)b * Hkv + kv) * (size_t)Lk * d;
    hc->lut = lut;
    hc->c_int = intattn_oracle_c_int(clip, s_q, s_k, d);
    return intattn_oracle_requant_params(s_v, s_o, &hc->rq_mult, &hc->rq_shift);
}

/*
 * Whole forward over the flattened (b * Hq + h) range [bh_begin, bh_end) and
 * the query rows [row_begin, row_end); everything outside is left untouched, so
 * a harness may fan disjoint ranges over host threads.
 *
 * q: [B,Hq,L,d]  k, v: [B,Hkv,Lk,d]  out: [B,Hq,L,d]   (contiguous, HOST pointers)
 * Lk != L: rectangular attention (a chunk of queries, or one decoded token, against a longer
 * key/value sequence); the causal mask is then aligned to the end and needs Lk >= L.
 * scale_mode 0: sq/sk/sv/so hold one float; 1: sq/so hold Hq floats, sk/sv hold Hkv.
 * so == NULL means s_O = s_V of the matching KV head.
 * Optional taps (NULL to skip): row_max, row_sum [B,Hq,L]; acc [B,Hq,L,d];
 * prob [B,Hq,L,Lk] (tiny problems only).
 */
int intattn_oracle_forward(int B, int Hq, int Hkv, int L, int Lk, int d, int causal, const int8_t *q,
                           const int8_t *k, const int8_t *v, int scale_mode, const float *sq,
                           const float *sk, const float *sv, const float *so, int lut_bits,
                           double clip, int bh_begin, int bh_end, int row_begin, int row_end,
                           int8_t *out, int32_t *row_max, int32_t *row_sum, int32_t *acc,
                           uint8_t *prob)
{
    int rc = check_problem(B, Hq, Hkv, L, Lk, causal, d, lut_bits, clip, q, k, v, sq, sk, sv);
    if (rc) return rc;
    if (!out || bh_begin < 0 || bh_end > B * Hq || row_begin < 0 || row_end > L) return ORACLE_BAD_ARG;

    uint8_t lut[256];
    rc = intattn_oracle_lut(lut_bits, clip, lut);
    if (rc) return rc;

    head_ctx hc;
    hc.a = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    hc.e = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    hc.p = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    if (!hc.a || !hc.e || !hc.p) {
        free(hc.a); free(hc.e); free(hc.p);
        return ORACLE_NO_MEM;
    }
    for (int bh = bh_begin; bh < bh_end && rc == ORACLE_OK; ++bh) {
        const int b = bh / Hq, hq = bh % Hq;
        rc = head_setup(&hc, Hq, Hkv, L, Lk, d, causal, b, hq, q, k, v, scale_mode, sq, sk, sv, so,
                        lut_bits, clip, lut);
        if (rc) break;
        for (int i = row_begin; i < row_end; ++i) {
            size_t row = (size_t)bh * L + i;
            oracle_row(&hc, i, out + row * d, row_max ? row_max + row : NULL,
                       row_sum ? row_sum + row : NULL, acc ? acc + row * d : NULL,
                       prob ? prob + row * Lk : NULL);
        }
    }
    free(hc.a); free(hc.e); free(hc.p);
    return rc;
}

/*
 * Selected query rows of one (b, hq): rows[0..n_rows).  Outputs are packed by
 * sample: out [n_rows, d], row_max / row_sum [n_rows], acc [n_rows, d].
 * Used to check full-size problems on sampled rows.
 */
int intattn_oracle_rows(int B, int Hq, int Hkv, int L, int Lk, int d, int causal, const int8_t *q,
                        const int8_t *k, const int8_t *v, int scale_mode, const float *sq,
                        const float *sk, const float *sv, const float *so, int lut_bits,
                        double clip, int b, int hq, int n_rows, const int32_t *rows, int8_t *out,
                        int32_t *row_max, int32_t *row_sum, int32_t *acc)
{
    int rc = check_problem(B, Hq, Hkv, L, Lk, causal, d, lut_bits, clip, q, k, v, sq, sk, sv);
    if (rc) return rc;
    if (!out || !rows || b < 0 || b >= B || hq < 0 || hq >= Hq || n_rows < 0) return ORACLE_BAD_ARG;

    uint8_t lut[256];
    rc = intattn_oracle_lut(lut_bits, clip, lut);
    if (rc) return rc;

    head_ctx hc;
    hc.a = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    hc.e = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    hc.p = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    if (!hc.a || !hc.e || !hc.p) {
        free(hc.a); free(hc.e); free(hc.p);
        return ORACLE_NO_MEM;
    }
    rc = head_setup(&hc, Hq, Hkv, L, Lk, d, causal, b, hq, q, k, v, scale_mode, sq, sk, sv, so,
                    lut_bits, clip, lut);
    for (int s = 0; s < n_rows && rc == ORACLE_OK; ++s) {
        int i = rows[s];
        if (i < 0 || i >= L) { rc = ORACLE_BAD_ARG; break; }
        oracle_row(&hc, i, out + (size_t)s * d, row_max ? row_max + s : NULL,
                   row_sum ? row_sum + s : NULL, acc ? acc + (size_t)s * d : NULL, NULL);
    }
    free(hc.a); free(hc.e); free(hc.p);
    return rc;
}

/* ------------------------------------------------------------------ groups over the key axis (Sec. 3.3) */

/*
 * Finer quantization groups over BOTH axes of the logit matrix (Sec. 3.3, "Quantization Scope and
 * Compatibility"): Q is quantized per block of q_block consecutive query rows, K per block of
 * k_block consecutive keys (k_block = 1: one scale per key, i.e. per output channel of Q.K^T --
 * "per-channel"; larger: "per-block"), V per KV head.  Every logit A_hat[i, j] then has the scale
 * of its (row block, key block) pair,
 *     alpha^(g) = s_Q^(g) s_K^(g) / sqrt(d),      c_int^(g) = round(c / alpha^(g))       (Sec. 3.3),
 * clipping, index map and table lookup are the per-tensor formulas with c_int^(g), and the row is
 * normalized once over all its keys ("summing contributions within each row").
 *
 * READING (the paper does not say how Delta_hat^(g) is formed when the groups of one row have
 * different scales; integer logits of different groups are not comparable): the row maximum is
 * taken over the DEQUANTIZED logits,
 *     M = max_j alpha^(g(j)) * A_hat[i, j]                 (one fp64 product per logit),
 * and each group measures its distances from the image of M in its own integer units,
 *     m^(g) = round(M / alpha^(g)),    Delta_hat^(g)[j] = max(m^(g) - A_hat[i, j], 0).
 * With equal scales this is m = rowMax(A_hat) and the per-tensor pipeline, bit for bit.
 * c_int^(g) above 2^30 is capped at 2^30 (a range limit of this build; it needs
 * s_Q s_K < 6.2e-9 sqrt(d)).  Scales must be finite and > 0.
 * PARITY UNPINNED by the paper for this reading; pinned to the per-tensor pipeline (equal scales),
 * to fp64 softmax of the dequantized logits, and to an exact-rational restatement.
 *
 * q [B,Hq,L,d]; k, v [B,Hkv,Lk,d]; sq, so [B,Hq,ceil(L/q_block)] (so may be NULL: s_O = s_V);
 * sk [B,Hkv,ceil(Lk/k_block)]; sv [Hkv].  Taps (NULL to skip): row_max_real [B,Hq,L] (M, fp64),
 * row_sum [B,Hq,L], acc [B,Hq,L,d], prob [B,Hq,L,Lk].
 */
int intattn_oracle_forward_groups(int B, int Hq, int Hkv, int L, int Lk, int d, int causal, const int8_t *q,
                                  const int8_t *k, const int8_t *v, int q_block, int k_block,
                                  const float *sq, const float *sk, const float *sv, const float *so,
                                  int lut_bits, double clip, int8_t *out, double *row_max_real,
                                  int32_t *row_sum, int32_t *acc, uint8_t *prob)
{
    int rc = check_problem(B, Hq, Hkv, L, Lk, causal, d, lut_bits, clip, q, k, v, sq, sk, sv);
    if (rc) return rc;
    if (!out || q_block < 1 || k_block < 1) return ORACLE_BAD_ARG;
    const int nqb = (L + q_block - 1) / q_block, nkb = (Lk + k_block - 1) / k_block;
    const int64_t top = ((int64_t)1 << lut_bits) - 1;
    const int64_t C_INT_CAP = (int64_t)1 << 30;
    uint8_t lut[256];
    rc = intattn_oracle_lut(lut_bits, clip, lut);
    if (rc) return rc;
    for (int64_t e = 0; e < (int64_t)B * Hq * nqb; ++e)
        if (!(sq[e] > 0.0f) || isinf(sq[e]) || (so && (!(so[e] > 0.0f) || isinf(so[e])))) return ORACLE_BAD_ARG;
    for (int64_t e = 0; e < (int64_t)B * Hkv * nkb; ++e)
        if (!(sk[e] > 0.0f) || isinf(sk[e])) return ORACLE_BAD_ARG;

    int64_t *a = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    int64_t *ev = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    int64_t *pv = (int64_t *)malloc(sizeof(int64_t) * (size_t)Lk);
    double *alpha = (double *)malloc(sizeof(double) * (size_t)Lk);
    if (!a || !ev || !pv || !alpha) {
        free(a); free(ev); free(pv); free(alpha);
        return ORACLE_NO_MEM;
    }
    const int grp = Hq / Hkv;
    for (int bh = 0; bh < B * Hq && rc == ORACLE_OK; ++bh) {
        const int b = bh / Hq, hq = bh % Hq, kv = hq / grp;
        const int8_t *qh = q + (size_t)bh * L * d;
        const int8_t *kh = k + ((size_t)b * Hkv + kv) * (size_t)Lk * d;
        const int8_t *vh = v + ((size_t)b * Hkv + kv) * (size_t)Lk * d;
        const float *skh = sk + ((size_t)b * Hkv + kv) * nkb;
        for (int i = 0; i < L && rc == ORACLE_OK; ++i) {
            const size_t row = (size_t)bh * L + i;
            const float s_q = sq[(size_t)bh * nqb + i / q_block];
            const float s_v = sv[kv];
            const float s_o = so ? so[(size_t)bh * nqb + i / q_block] : s_v;
            int64_t rq_mult;
            int32_t rq_shift;
            rc = intattn_oracle_requant_params(s_v, s_o, &rq_mult, &rq_shift);
            if (rc) break;
            const int n_vis = causal ? (i + (Lk - L) + 1) : Lk;

            /* Eq. logit-scale, and the scale of every logit (Sec. 3.3) */
            for (int j = 0; j < n_vis; ++j) {
                int64_t s = 0;
                for (int c = 0; c < d; ++c) s += (int64_t)qh[(size_t)i * d + c] * (int64_t)kh[(size_t)j * d + c];
                a[j] = s;
                alpha[j] = ((double)s_q * (double)skh[j / k_block]) / sqrt((double)d);
            }
            /* row maximum of the dequantized logits */
            double M = alpha[0] * (double)a[0];
            for (int j = 1; j < n_vis; ++j) {
                const double x = alpha[j] * (double)a[j];
                if (x > M) M = x;
            }
            /* group-wise distance, clipping (Sec. 3.3), index map, Eq. gather16, rowSum */
            int64_t S = 0;
            for (int j = 0; j < n_vis; ++j) {
                double cd = floor(clip / alpha[j] + 0.5);
                int64_t c_int = !(cd >= 1.0) ? 1 : (cd > (double)C_INT_CAP ? C_INT_CAP : (int64_t)cd);
                double md = floor(M / alpha[j] + 0.5); /* image of the row maximum in this group's units */
                if (md > 4.0e18) md = 4.0e18;
                if (md < -4.0e18) md = -4.0e18;
                int64_t delta = (int64_t)md - a[j];
                if (delta < 0) delta = 0;
                const int64_t dclip = delta < c_int ? delta : c_int;
                const int64_t idx = round_div(dclip * top, c_int);
                ev[j] = (int64_t)lut[idx];
                S += ev[j];
            }
            /* Eq. uint8-prob over the whole row */
            for (int j = 0; j < n_vis; ++j) pv[j] = intattn_oracle_prob(ev[j], S);
            if (prob)
                for (int j = 0; j < Lk; ++j) prob[row * Lk + j] = (j < n_vis) ? (uint8_t)pv[j] : 0;
            if (row_max_real) row_max_real[row] = M;
            if (row_sum) row_sum[row] = (int32_t)S;
            /* P_hat * V_hat, requantization */
            const int64_t half = (int64_t)1 << (rq_shift - 1), den = (int64_t)1 << rq_shift;
            for (int c = 0; c < d; ++c) {
                int64_t s = 0;
                for (int j = 0; j < n_vis; ++j) s += pv[j] * (int64_t)vh[(size_t)j * d + c];
                if (acc) acc[row * d + c] = (int32_t)s;
                int64_t o = floor_div(s * rq_mult + half, den);
                if (o > 127) o = 127;
                if (o < -127) o = -127;
                out[row * d + c] = (int8_t)o;
            }
        }
    }
    free(a); free(ev); free(pv); free(alpha);
    return rc;
}

/* ------------------------------------------------------------------ IndexSoftmax as an operator */

/*
 * IndexSoftmax (Sec. 3.1-3.2) on caller-supplied INT32 logits, the paper's softmax-only setting:
 * for every row  m = max, Delta = m - A, Delta' = min(Delta, c_int)  (Eq. int_clipping),
 * idx = round(Delta' (2^b - 1) / c_int), E = LUT_hat[idx]  (Eq. gather16), S = rowSum(E),
 * P = round(255 E / S)  (Eq. uint8-prob).
 * logits, prob: [rows, cols] contiguous.  rows_per_matrix > 0 with causal = 1 treats the rows as
 * stacked [rows_per_matrix, cols] matrices with the mask of the attention path (row r of a matrix
 * sees columns j <= r + cols - rows_per_matrix; hidden columns get P = 0); otherwise every column
 * is visible.
 */
int intattn_oracle_index_softmax(int64_t rows, int64_t cols, const int32_t *logits, int64_t c_int,
                                 int lut_bits, double clip, int64_t rows_per_matrix, int causal,
                                 uint8_t *prob)
{
    if (rows < 1 || cols < 1 || !logits || !prob || c_int < 1) return ORACLE_BAD_ARG;
    if (causal && (rows_per_matrix < 1 || cols < rows_per_matrix || rows % rows_per_matrix != 0)) return ORACLE_BAD_ARG;
    uint8_t lut[256];
    int rc = intattn_oracle_lut(lut_bits, clip, lut);
    if (rc) return rc;
    int64_t *e = (int64_t *)malloc(sizeof(int64_t) * (size_t)cols);
    if (!e) return ORACLE_NO_MEM;
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t *a = logits + r * cols;
        const int64_t n_vis = causal ? (r % rows_per_matrix) + (cols - rows_per_matrix) + 1 : cols;
        int64_t m = a[0];
        for (int64_t j = 1; j < n_vis; ++j)
            if (a[j] > m) m = a[j];
        int64_t S = 0;
        for (int64_t j = 0; j < n_vis; ++j) {
            int64_t delta = m - (int64_t)a[j];
            int64_t dclip = delta < c_int ? delta : c_int;
            e[j] = (int64_t)lut[intattn_oracle_index(dclip, c_int, lut_bits)];
            S += e[j];
        }
        for (int64_t j = 0; j < cols; ++j) prob[r * cols + j] = j < n_vis ? (uint8_t)intattn_oracle_prob(e[j], S) : 0;
    }
    free(e);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ dynamic quantizer (Sec. 2.1) */

/* Eq. quant: s_X = max|X| / 127, quant(X) = clamp(round(X / s_X), -127, 127), symmetric, zero
 * point 0.  x is [B, H, L, d] contiguous fp32 (fp16 / bf16 inputs are widened exactly by the
 * caller).  per_head = 0: one scale for the tensor (the paper's per-tensor form); 1: one scale
 * per head index (axis 1) shared over the batch (Sec. 3.3 with one group per head).
 * scales receives 1 or H values.  Inputs must be finite. */
int intattn_oracle_quantize(int B, int H, int L, int d, const float *x, int per_head, int8_t *xq,
                            float *scales)
{
    if (B < 1 || H < 1 || L < 1 || d < 1 || !x || !xq || !scales) return ORACLE_BAD_ARG;
    const int groups = per_head ? H : 1;
    const int64_t head_elems = (int64_t)L * d;
    for (int g = 0; g < groups; ++g) {
        float amax = 0.0f;
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h) {
                if (per_head && h != g) continue;
                const float *xs = x + ((int64_t)b * H + h) * head_elems;
                for (int64_t i = 0; i < head_elems; ++i) {
                    const float a = fabsf(xs[i]);
                    if (a > amax) amax = a;
                }
            }
        if (amax < 1e-12f) amax = 1e-12f;
        scales[g] = amax / 127.0f; /* one fp32 division */
    }
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const float s = scales[per_head ? h : 0];
            const float *xs = x + ((int64_t)b * H + h) * head_elems;
            int8_t *qs = xq + ((int64_t)b * H + h) * head_elems;
            for (int64_t i = 0; i < head_elems; ++i) {
                float r = rintf(xs[i] / s); /* fp32 division, nearest integer, ties to even */
                if (r > 127.0f) r = 127.0f;
                if (r < -127.0f) r = -127.0f;
                qs[i] = (int8_t)r;
            }
        }
    return ORACLE_OK;
}
