// Host side of the C ABI declared in include/intattn.h: argument checking, derivation of the
// integer parameters from the scales (Eq. logit-scale, Eq. clipping_thr), LUT_hat
// (Eq. lut_re, Eq. lut16), and kernel launches.  No CPU fallback exists: if a launch
// fails, the error is returned.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/intattn.h"
#include "params.h"

using namespace intattn;

// Workspace of intattn_forward_noalloc: one array per GPU in the library's image.  The name below is
// a host-side stand-in, not a device address: every use goes through the pointer that
// hipGetSymbolAddress returned for the device at hand (g_scratch_ptr).
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)INTATTN_NOALLOC_SCRATCH_BYTES;
constexpr size_t STATIC_TABLE_BYTES = 16384; // head of the scratch: per-head parameter table (512 heads)
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES] = {nullptr};
static std::mutex g_scratch_mu;

// Pinned host staging for small host-to-device uploads (per-head tables): the bytes are copied here
// first, so the asynchronous copy never reads memory that the caller, or a returning function, owns.
struct Staging {
    unsigned char *host = nullptr;
    hipEvent_t done = nullptr;
    bool pending = false;
};
constexpr size_t STAGING_BYTES = 65536;

struct intattn_ctx {
    int device = 0;
    int lut_bits = 5;
    double clip = 6.6;
    int variant = 0;
    uint8_t lut[64] = {0};
    // device-side per-head tables (allocated on first per-head call, grown on demand)
    HeadParams *d_hp = nullptr;
    float *d_alpha = nullptr, *d_svso = nullptr;
    int table_cap = 0;
    // kernel workspace (row max and row sum between the two launches, V chunk sums), grown on demand
    int32_t *d_ws = nullptr;
    size_t ws_cap = 0; // in int32 elements
    HeadParams *d_rowtab = nullptr; // parameters per block of query rows (scale_mode 2), grown on demand
    uint32_t *d_dec_state = nullptr; // fused split-key kernel: DEC_STATE_WORDS per (batch, KV head) group, zero between launches
    size_t dec_state_groups = 0;
    size_t rowtab_cap = 0;
    int32_t *d_status = nullptr; // per head: what the last derivation on the device found (intattn_dynamic_status)
    int status_cap = 0, status_n = 0;
    float *d_amax = nullptr; // scratch of the quantizer: partial max|X| per workgroup of its first pass
    int64_t amax_cap = 0;
    // parameters derived from the host scales of the last call (the search for index-map constants costs
    // microseconds per head; serving loops pass the same scales again and again)
    std::vector<uint32_t> dv_key;
    std::vector<HeadParams> dv_hp;
    std::vector<HeadParams> dv_hp_c;
    std::vector<float> dv_alpha, dv_svso;
    int dv_mode = 0;
    std::vector<HeadParams> hp_host;  // what d_hp currently holds
    std::vector<float> alpha_host, svso_host;
    Staging stage[2];
    int stage_next = 0;
    std::string err;
};

namespace {

thread_local std::string g_create_err;

int fail(intattn_ctx *ctx, int code, const std::string &msg)
{
    if (ctx) ctx->err = msg;
    else g_create_err = msg;
    return code;
}

int hip_fail(intattn_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, INTATTN_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Stream-ordered upload of a small table through the context's pinned staging buffers.  Two slots
// alternate; a slot is reused only after the copy that last read it has completed (an event per
// slot), so the call blocks only when more than two uploads are in flight -- tables change rarely.
int upload(intattn_ctx *ctx, void *dst, const void *src, size_t bytes, hipStream_t st, const char *what)
{
    if (bytes > STAGING_BYTES) return fail(ctx, INTATTN_ERR_UNSUPPORTED, std::string(what) + ": table exceeds the staging buffer");
    Staging &sg = ctx->stage[ctx->stage_next];
    ctx->stage_next ^= 1;
    if (!sg.host) return fail(ctx, INTATTN_ERR_NOMEM, "no staging buffer (host-only context)");
    if (sg.pending) {
        const hipError_t e = hipEventSynchronize(sg.done);
        if (e != hipSuccess) return hip_fail(ctx, e, "hipEventSynchronize(staging)");
        sg.pending = false;
    }
    std::memcpy(sg.host, src, bytes);
    hipError_t e = hipMemcpyAsync(dst, sg.host, bytes, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipEventRecord(sg.done, st);
    if (e != hipSuccess) return hip_fail(ctx, e, what);
    sg.pending = true;
    return INTATTN_OK;
}

// Scoped "make ctx->device current", restoring the caller's device afterwards.
struct DeviceGuard {
    int prev = -1;
    bool changed = false;
    hipError_t status = hipSuccess;
    explicit DeviceGuard(int dev)
    {
        status = hipGetDevice(&prev);
        if (status == hipSuccess && prev != dev) {
            status = hipSetDevice(dev);
            changed = (status == hipSuccess);
        }
    }
    ~DeviceGuard()
    {
        if (changed) (void)hipSetDevice(prev);
    }
};

bool good_scale(float s) { return std::isfinite(s) && s > 0.0f; }

// Eq. clipping_thr.  Capped at 2^30: with |A_hat| <= 128*128*d the index is 0 for every
// element once c_int > 62 * 2 * 128*128*128, so the cap never changes a result.
int64_t derive_c_int(double clip, float s_q, float s_k, int d)
{
    const double alpha = ((double)s_q * (double)s_k) / std::sqrt((double)d);
    const double c = std::floor(clip / alpha + 0.5);
    if (!(c >= 1.0)) return 1;
    if (c > 1073741824.0) return 1073741824LL;
    return (int64_t)c;
}

bool derive_requant(float s_v, float s_o, int32_t *mult, int32_t *shift)
{
    const double r = (double)s_v / (255.0 * (double)s_o);
    if (!(r > 0.0) || !std::isfinite(r)) return false;
    int e = 0;
    const double m = std::frexp(r, &e);
    long long M = std::llround(m * 2147483648.0);
    if (M == 2147483648LL) {
        M = 1073741824LL;
        e += 1;
    }
    const int sh = 31 - e;
    if (sh < 1 || sh > 62) return false;
    *mult = (int32_t)M;
    *shift = sh;
    return true;
}

uint32_t true_index(uint64_t dclip, uint64_t c_int, uint64_t top) { return (uint32_t)((2 * top * dclip + c_int) / (2 * c_int)); }

// Check points for a candidate index map: both the exact map and every candidate are
// monotone step functions of x, so agreement at x = 0, x = c_int and on both sides of every
// true step proves agreement on the whole range [0, c_int].
std::vector<uint32_t> check_points(uint32_t c_int, uint32_t top)
{
    std::vector<uint32_t> pts;
    pts.push_back(0);
    pts.push_back(c_int);
    for (uint64_t k = 1; k <= top; ++k) {
        // smallest x with round(x*top/c_int) >= k:  x >= (2k-1) c_int / (2 top)
        const uint64_t num = (2 * k - 1) * (uint64_t)c_int, den = 2ull * top;
        const uint64_t t = (num + den - 1) / den;
        if (t <= c_int) {
            pts.push_back((uint32_t)t);
            if (t > 0) pts.push_back((uint32_t)(t - 1));
        }
    }
    return pts;
}

// Finds (mul, add, shift) with ((x * mul + add) >> shift) == round(x * top / c_int) for every
// integer x in [0, c_int], with signed 24-bit factors and a sum below 2^31.
// Stored for the kernel as idx_mul = -mul (the kernel multiplies t = -x), idx_add = add.
bool find_mad24(uint32_t c_int, uint32_t top, HeadParams *hp)
{
    if (c_int >= (1u << 23)) return false;
    const std::vector<uint32_t> pts = check_points(c_int, top);
    for (int s = 27; s >= 8; --s) {
        const uint64_t num = (uint64_t)top << s;
        const uint64_t cands[2] = {(num + c_int - 1) / c_int, num / c_int};
        for (uint64_t mul : cands) {
            if (mul == 0 || mul >= (1ull << 23)) continue;
            const uint64_t add = 1ull << (s - 1);
            if ((uint64_t)c_int * mul + add >= (1ull << 31)) continue;
            bool ok = true;
            for (uint32_t x : pts) {
                const uint32_t got = (uint32_t)(((uint64_t)x * mul + add) >> s);
                if (got != true_index(x, c_int, top)) {
                    ok = false;
                    break;
                }
            }
            if (ok) {
                hp->idx_mul = (uint32_t)(-(int32_t)mul);
                hp->idx_add = (uint32_t)add;
                hp->idx_shift = s;
                return true;
            }
        }
    }
    return false;
}

// The MAD24 form with the shift fixed at 24, so that the index is the top byte of x * mul + add (the
// sum stays below 2^30): mul ~ top * 2^24 / c_int, and every check point x with exact index k confines
// add to k * 2^24 <= x * mul + add < (k + 1) * 2^24.  Exists for thresholds from about 2 * top up to
// several thousand (beyond that a 24-bit fraction no longer separates the steps).
// Stored as idx_mul = -mul, idx_add = add, idx_shift = 24.
bool find_top24(uint32_t c_int, uint32_t top, HeadParams *hp)
{
    if (c_int >= (1u << 23)) return false;
    const std::vector<uint32_t> pts = check_points(c_int, top);
    const int64_t m0 = (int64_t)(((uint64_t)top << 24) / c_int);
    for (int64_t dm = 0; dm < 40; ++dm) {
        for (int sgn = 0; sgn < 2; ++sgn) {
            const int64_t mul = sgn ? m0 - dm : m0 + 1 + dm;
            if (mul < 1 || mul >= (1ll << 23)) continue;
            int64_t lo = 0, hi = (1ll << 31) - 1 - (int64_t)c_int * mul;
            for (uint32_t x : pts) {
                const int64_t k = (int64_t)true_index(x, c_int, top);
                const int64_t need_lo = (k << 24) - (int64_t)x * mul, need_hi = ((k + 1) << 24) - 1 - (int64_t)x * mul;
                if (need_lo > lo) lo = need_lo;
                if (need_hi < hi) hi = need_hi;
                if (lo > hi) break;
            }
            if (lo > hi) continue;
            hp->idx_mul = (uint32_t)(-(int32_t)mul);
            hp->idx_add = (uint32_t)(lo + (hi - lo) / 2);
            hp->idx_shift = 24;
            return true;
        }
    }
    return false;
}

// Finds (pre, off, mul) with ((((x << pre) + off) * mul) >> 32) == round(x * top / c_int) for
// every integer x in [0, c_int], where (x << pre) + off and mul stay below 2^23 so that the
// 48-bit product of two signed 24-bit factors is exact.  mul ~ top * 2^(32-pre) / c_int and
// off ~ 2^31 / mul (half an index step).
// Stored for the kernel as idx_mul = -mul, idx_add = -off (it works on t = -x), idx_shift = pre.
bool find_mulhi24(uint32_t c_int, uint32_t top, HeadParams *hp)
{
    const std::vector<uint32_t> pts = check_points(c_int, top);
    for (int pre = 0; pre <= 22; ++pre) {
        if (((uint64_t)c_int << pre) >= (1ull << 23)) break;
        const long double ideal = (long double)top * 4294967296.0L / ((long double)c_int * (long double)(1ull << pre));
        if (ideal >= 8388607.0L) continue; // multiplier too wide: shift x further left
        if (ideal < 1024.0L) break;
        const int64_t m0 = (int64_t)ideal;
        for (int64_t dm = 0; dm <= 16; ++dm) {
            for (int sgn = 0; sgn < 2; ++sgn) {
                const int64_t mul = sgn ? m0 - dm : m0 + 1 + dm;
                if (mul < 1 || mul >= (1ll << 23)) continue;
                // every check point x with exact index k confines off to
                //   k*2^32 <= ((x << pre) + off) * mul < (k+1)*2^32
                int64_t lo = 0, hi = (1ll << 23) - 1 - ((int64_t)c_int << pre);
                for (uint32_t x : pts) {
                    const int64_t k = (int64_t)true_index(x, c_int, top);
                    const int64_t xs = (int64_t)x << pre;
                    const int64_t need_lo = (k * 4294967296LL + mul - 1) / mul - xs;
                    const int64_t need_hi = ((k + 1) * 4294967296LL - 1) / mul - xs;
                    if (need_lo > lo) lo = need_lo;
                    if (need_hi < hi) hi = need_hi;
                    if (lo > hi) break;
                }
                if (lo > hi) continue;
                const int64_t off = lo + (hi - lo) / 2;
                hp->idx_mul = (uint32_t)(-(int32_t)mul);
                hp->idx_add = (uint32_t)(-(int32_t)off);
                hp->idx_shift = pre;
                return true;
            }
        }
    }
    return false;
}

// Finds an fp32 factor r ~ top / c_int with trunc(fma(-x, -r, 0.5)) == round(x * top / c_int)
// for every integer x in [0, c_int] (c_int < 2^24 so that x is exact in fp32).  The check runs
// the same IEEE single-precision fma the kernel runs.  Stored as idx_mul = bits of -r.
bool find_fp32(uint32_t c_int, uint32_t top, HeadParams *hp)
{
    if (c_int >= (1u << 24)) return false;
    const std::vector<uint32_t> pts = check_points(c_int, top);
    float r = (float)((double)top / (double)c_int);
    r = std::nextafterf(r, 0.0f);
    for (int step = 0; step < 3; ++step, r = std::nextafterf(r, 1e30f)) {
        bool ok = true;
        for (uint32_t x : pts) {
            const float y = std::fmaf(-(float)x, -r, 0.5f);
            if ((uint32_t)(int)y != true_index(x, c_int, top)) {
                ok = false;
                break;
            }
        }
        if (ok) {
            const float negr = -r;
            std::memcpy(&hp->idx_mul, &negr, 4);
            hp->idx_add = 0;
            hp->idx_shift = 0;
            return true;
        }
    }
    return false;
}

// The fp64 scheme: r = the double after fl(top / c_int); idx = trunc(fma(x, r, 0.5)) in IEEE double.
// Exact for every c_int <= 2^30 and x <= c_int without a search: r exceeds top/c_int by less than
// two units in the last place, so y = x*r + 0.5 exceeds v = x*top/c_int + 0.5 by less than 2^-43
// before and 2^-42 after the rounding of the fma, which is monotone: an integer v = k (a tie of the
// rounding to nearest index) stays >= k, and any other v lies at least 1/(2 c_int) >= 2^-31 below
// the next integer.  The check points are evaluated all the same.
// Stored for the kernel as the bits of -r: low word in idx_mul, high word in idx_add.
bool find_fp64(uint32_t c_int, uint32_t top, HeadParams *hp)
{
    const double r = std::nextafter((double)top / (double)c_int, 1e300);
    for (uint32_t x : check_points(c_int, top))
        if ((uint32_t)(int)std::fma(-(double)x, -r, 0.5) != true_index(x, c_int, top)) return false;
    const double negr = -r;
    uint64_t bits;
    std::memcpy(&bits, &negr, 8);
    hp->idx_mul = (uint32_t)bits;
    hp->idx_add = (uint32_t)(bits >> 32);
    hp->idx_shift = 0;
    return true;
}

struct Derived {
    std::vector<HeadParams> hp;
    std::vector<HeadParams> hp_c; // per head, for sweep C alone: top-byte constants where they exist (pad[0] names the scheme); empty: as hp
    std::vector<float> alpha, svso;
    int idx_mode = IDX_MAD24;
};

int validate(intattn_ctx *ctx, const intattn_args *a)
{
    if (!ctx) return INTATTN_ERR_INVALID_ARG;
    if (!a) return fail(ctx, INTATTN_ERR_INVALID_ARG, "args is NULL");
    if (a->B < 1 || a->Hq < 1 || a->Hkv < 1 || a->L < 1)
        return fail(ctx, INTATTN_ERR_INVALID_ARG, "B, Hq, Hkv, L must be >= 1");
    if (a->Hq % a->Hkv != 0) return fail(ctx, INTATTN_ERR_INVALID_ARG, "Hq must be a multiple of Hkv");
    if (a->d != 64 && a->d != 128) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "d must be 64 or 128");
    if (a->L > 131071) return fail(ctx, INTATTN_ERR_INVALID_ARG, "L exceeds 131071 (int32 accumulator bound)");
    if (a->Lkv < 0 || a->Lkv > 131071) return fail(ctx, INTATTN_ERR_INVALID_ARG, "Lkv must be 0 (= L) or in 1..131071 (int32 accumulator bound)");
    const int Lk = a->Lkv ? a->Lkv : a->L;
    if (a->causal == 1 && Lk < a->L)
        return fail(ctx, INTATTN_ERR_INVALID_ARG, "a causal mask needs Lkv >= L (it is aligned to the end of the keys)");
    if (a->causal != 0 && a->causal != 1) return fail(ctx, INTATTN_ERR_INVALID_ARG, "causal must be 0 or 1");
    if (a->scale_mode < 0 || a->scale_mode > 3) return fail(ctx, INTATTN_ERR_INVALID_ARG, "scale_mode must be 0, 1, 2 or 3");
    if (a->scale_mode >= 2 && a->q_block < 1) return fail(ctx, INTATTN_ERR_INVALID_ARG, "scale_mode 2 and 3 need q_block >= 1");
    if (a->scale_mode == 3 && a->k_block < 1) return fail(ctx, INTATTN_ERR_INVALID_ARG, "scale_mode 3 needs k_block >= 1");
    if (a->scale_mode != 3 && a->k_block != 0) return fail(ctx, INTATTN_ERR_INVALID_ARG, "k_block must be 0 unless scale_mode is 3");
    if (!a->q || !a->k || !a->v || !a->out) return fail(ctx, INTATTN_ERR_INVALID_ARG, "q, k, v, out must be non-NULL");
    if (!a->scale_q || !a->scale_k || !a->scale_v)
        return fail(ctx, INTATTN_ERR_INVALID_ARG, "scale_q, scale_k, scale_v must be non-NULL");
    if ((const void *)a->out == (const void *)a->q || (const void *)a->out == (const void *)a->k ||
        (const void *)a->out == (const void *)a->v)
        return fail(ctx, INTATTN_ERR_INVALID_ARG, "out must not alias an input");
    const void *ptrs[4] = {a->q, a->k, a->v, a->out};
    for (const void *ptr : ptrs)
        if (((uintptr_t)ptr & 15u) != 0) return fail(ctx, INTATTN_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    const int64_t *strides[4] = {a->q_stride, a->k_stride, a->v_stride, a->out_stride};
    for (const int64_t *s : strides) {
        for (int i = 0; i < 3; ++i)
            if (s[i] < 0 || (s[i] & 15) != 0)
                return fail(ctx, INTATTN_ERR_INVALID_ARG, "strides must be non-negative multiples of 16");
        if (s[2] < a->d) return fail(ctx, INTATTN_ERR_INVALID_ARG, "the L stride must be at least d");
        if (s[2] > (1 << 24)) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "the L stride must not exceed 2^24 bytes");
    }
    const int64_t rows_per_block = fwd_rows_per_block(fwd_choose_variant(ctx->variant, a->B, a->Hq, a->L, Lk, a->d, a->causal));
    const int64_t n_qtiles = fwd_row_tiles(a->causal == 1 ? Lk - a->L : 0, a->L, (int)rows_per_block);
    // the launch grid pads the (batch, KV head) groups to a multiple of the 8 XCDs
    const int64_t groups_padded = (((int64_t)a->B * a->Hkv + 7) / 8) * 8;
    if (n_qtiles * groups_padded * (int64_t)(a->Hq / a->Hkv) > 2147483647LL)
        return fail(ctx, INTATTN_ERR_UNSUPPORTED, "problem needs more than 2^31-1 workgroups");
    return INTATTN_OK;
}

int derive_all(intattn_ctx *ctx, const intattn_args *a, Derived *out)
{
    const int n = a->scale_mode ? a->Hq : 1;
    const int g = a->Hq / a->Hkv;
    const uint32_t top = (1u << ctx->lut_bits) - 1u;
    out->hp.assign((size_t)n, HeadParams{});
    out->alpha.assign((size_t)n, 0.f);
    out->svso.assign((size_t)n, 0.f);
    // candidate index-map schemes in order of preference; a launch uses one scheme for all heads
    typedef bool (*finder)(uint32_t, uint32_t, HeadParams *);
    const finder finders[5] = {find_top24, find_mulhi24, find_mad24, find_fp32, find_fp64};
    const int modes[5] = {IDX_TOP24, IDX_MULHI24, IDX_MAD24, IDX_FP32, IDX_FP64};
    bool all_ok[5] = {true, true, true, true, true};
    std::vector<HeadParams> cand[5];
    for (auto &c : cand) c.assign((size_t)n, HeadParams{});
    std::vector<char> top_ok((size_t)n, 0);
    for (int h = 0; h < n; ++h) {
        const int kv = a->scale_mode ? h / g : 0;
        const float sq = a->scale_q[h], sk = a->scale_k[kv], sv = a->scale_v[kv];
        const float so = a->scale_out ? a->scale_out[h] : sv;
        if (!good_scale(sq) || !good_scale(sk) || !good_scale(sv) || !good_scale(so))
            return fail(ctx, INTATTN_ERR_INVALID_ARG, "scales must be finite and > 0");
        HeadParams &hp = out->hp[(size_t)h];
        hp.c_int = (int32_t)derive_c_int(ctx->clip, sq, sk, a->d);
        if (!derive_requant(sv, so, &hp.rq_mult, &hp.rq_shift))
            return fail(ctx, INTATTN_ERR_INVALID_ARG, "s_V / (255 s_O) is outside the representable range");
        for (int m = 0; m < 5; ++m) {
            cand[m][(size_t)h] = hp;
            if (m == 0) { // the top-byte scheme: per head, for the mixed table of sweep C
                top_ok[(size_t)h] = finders[0]((uint32_t)hp.c_int, top, &cand[0][(size_t)h]);
                if (!top_ok[(size_t)h]) all_ok[0] = false;
            } else if (all_ok[m] && !finders[m]((uint32_t)hp.c_int, top, &cand[m][(size_t)h])) {
                all_ok[m] = false;
            }
        }
        out->alpha[(size_t)h] = (float)(((double)sq * (double)sk) / std::sqrt((double)a->d));
        out->svso[(size_t)h] = (float)((double)sv / (double)so);
    }
    for (int m = 0; m < 5; ++m) {
        if (all_ok[m]) {
            out->idx_mode = modes[m];
            out->hp = cand[m];
            out->hp_c.clear();
            // Some heads only lack top-byte constants (thresholds below 62 or of many thousands): sweep C, where that
            // scheme saves a vector instruction per score, then takes each head's own scheme from a table of its own.
            int n_top = 0;
            for (int h = 0; h < n; ++h) n_top += top_ok[(size_t)h] ? 1 : 0;
            if (modes[m] == IDX_MULHI24 && n > 1 && n_top > 0) {
                out->hp_c = cand[m];
                for (int h = 0; h < n; ++h) {
                    if (top_ok[(size_t)h]) out->hp_c[(size_t)h] = cand[0][(size_t)h];
                    out->hp_c[(size_t)h].pad[0] = top_ok[(size_t)h] ? IDX_TOP24 : IDX_MULHI24;
                }
            }
            return INTATTN_OK;
        }
    }
    return fail(ctx, INTATTN_ERR_UNSUPPORTED, "no exact index map for these scales");
}

int ensure_tables(intattn_ctx *ctx, int n)
{
    if (n <= ctx->table_cap) return INTATTN_OK;
    int cap = ctx->table_cap ? ctx->table_cap : 64;
    while (cap < n) cap *= 2;
    HeadParams *hp = nullptr;
    float *al = nullptr, *sv = nullptr;
    hipError_t e = hipMalloc((void **)&hp, sizeof(HeadParams) * (size_t)cap);
    if (e == hipSuccess) e = hipMalloc((void **)&al, sizeof(float) * (size_t)cap);
    if (e == hipSuccess) e = hipMalloc((void **)&sv, sizeof(float) * (size_t)cap);
    if (e != hipSuccess) {
        if (hp) (void)hipFree(hp);
        if (al) (void)hipFree(al);
        if (sv) (void)hipFree(sv);
        return fail(ctx, INTATTN_ERR_NOMEM, std::string("hipMalloc of per-head tables: ") + hipGetErrorString(e));
    }
    // Frees are stream-ordered with respect to earlier work in HIP (the free waits), so old
    // tables that a running kernel may still read are released safely.
    if (ctx->d_hp) (void)hipFree(ctx->d_hp);
    if (ctx->d_alpha) (void)hipFree(ctx->d_alpha);
    if (ctx->d_svso) (void)hipFree(ctx->d_svso);
    ctx->d_hp = hp;
    ctx->d_alpha = al;
    ctx->d_svso = sv;
    ctx->table_cap = cap;
    ctx->hp_host.clear();
    ctx->alpha_host.clear();
    ctx->svso_host.clear();
    return INTATTN_OK;
}

int ensure_workspace(intattn_ctx *ctx, size_t n_int32)
{
    if (n_int32 <= ctx->ws_cap) return INTATTN_OK;
    int32_t *ws = nullptr;
    const hipError_t e = hipMalloc((void **)&ws, n_int32 * sizeof(int32_t));
    if (e != hipSuccess)
        return fail(ctx, INTATTN_ERR_NOMEM, std::string("hipMalloc of the kernel workspace: ") + hipGetErrorString(e));
    if (ctx->d_ws) (void)hipFree(ctx->d_ws); // hipFree waits for work that may still read it
    ctx->d_ws = ws;
    ctx->ws_cap = n_int32;
    return INTATTN_OK;
}

// What a call may do beyond the plain forward.
struct RunMode {
    bool comparator = false; // the conventional INT8 pipeline instead of the integer one
    int stage = 0;           // 0: everything; 1 / 2: the two launches of the tiled path separately
    bool dynamic = false;    // the scale pointers of the arguments are DEVICE memory: parameters derived by a kernel
    bool no_alloc = false;   // workspace and per-head table in the static device array; nothing is allocated
    bool reserve = false;    // allocate what the call would need and return without deriving or launching
};

int run(intattn_ctx *ctx, const intattn_args *a, void *stream, const RunMode &rm)
{
    const bool comparator = rm.comparator, dynamic = rm.dynamic;
    const int stage = rm.stage;
    int rc = validate(ctx, a);
    if (rc) return rc;
    if (ctx->device < 0) return fail(ctx, INTATTN_ERR_INVALID_ARG, "host-only context (device -1) cannot launch");
    if (a->scale_mode >= 2 && (!dynamic || comparator))
        return fail(ctx, INTATTN_ERR_UNSUPPORTED, "scale_mode 2 and 3 (groups of query rows / of keys) are served by intattn_forward_dynamic only");
    if (a->scale_mode == 3 && stage != 0)
        return fail(ctx, INTATTN_ERR_UNSUPPORTED, "scale_mode 3 runs in a single launch: no stages");
    Derived dv;
    if (dynamic) {
        dv.idx_mode = a->scale_mode == 3 ? IDX_KGROUP : (a->scale_mode == 2 ? IDX_ROW64 : IDX_DEVICE);
    } else if (!rm.reserve) {
        // everything the derivation depends on, bit for bit
        const int n_q = a->scale_mode ? a->Hq : 1, n_kv = a->scale_mode ? a->Hkv : 1;
        std::vector<uint32_t> key;
        key.reserve(5 + 2 * (size_t)n_q + 2 * (size_t)n_kv);
        const uint32_t head[5] = {(uint32_t)a->scale_mode, (uint32_t)a->d, (uint32_t)a->Hq, (uint32_t)a->Hkv, a->scale_out ? 1u : 0u};
        key.insert(key.end(), head, head + 5);
        auto add = [&](const float *x, int n) {
            for (int i = 0; i < n; ++i) {
                uint32_t bits;
                std::memcpy(&bits, x + i, 4);
                key.push_back(bits);
            }
        };
        add(a->scale_q, n_q);
        add(a->scale_k, n_kv);
        add(a->scale_v, n_kv);
        if (a->scale_out) add(a->scale_out, n_q);
        if (!ctx->dv_key.empty() && key == ctx->dv_key) {
            dv.hp = ctx->dv_hp;
            dv.hp_c = ctx->dv_hp_c;
            dv.alpha = ctx->dv_alpha;
            dv.svso = ctx->dv_svso;
            dv.idx_mode = ctx->dv_mode;
        } else {
            rc = derive_all(ctx, a, &dv);
            if (rc) return rc;
            ctx->dv_key = key;
            ctx->dv_hp = dv.hp;
            ctx->dv_hp_c = dv.hp_c;
            ctx->dv_alpha = dv.alpha;
            ctx->dv_svso = dv.svso;
            ctx->dv_mode = dv.idx_mode;
        }
    }

    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return hip_fail(ctx, guard.status, "hipSetDevice");
    hipStream_t st = (hipStream_t)stream;

    // device memory of the call: the context's (allocated on demand), or the static array of this GPU
    unsigned char *static_base = nullptr;
    if (rm.no_alloc) {
        if (ctx->device >= MAX_DEVICES || !(static_base = (unsigned char *)g_scratch_ptr[ctx->device]))
            return fail(ctx, INTATTN_ERR_HIP, "the static workspace of this device was not resolved at intattn_create");
    }
    HeadParams *d_hp = nullptr; // per-head parameter table in use
    auto get_tables = [&](int n) -> int {
        if (rm.no_alloc) {
            if ((size_t)n * sizeof(HeadParams) > STATIC_TABLE_BYTES)
                return fail(ctx, INTATTN_ERR_UNSUPPORTED, "intattn_forward_noalloc: more than 512 query heads with per-head scales");
            d_hp = (HeadParams *)static_base;
            return INTATTN_OK;
        }
        const int r = ensure_tables(ctx, n);
        d_hp = ctx->d_hp;
        return r;
    };
    int32_t *d_ws = nullptr; // kernel workspace in use
    auto get_ws = [&](size_t n_int32) -> int {
        if (rm.no_alloc) {
            if (n_int32 * sizeof(int32_t) > STATIC_SCRATCH_BYTES - STATIC_TABLE_BYTES)
                return fail(ctx, INTATTN_ERR_UNSUPPORTED,
                            "intattn_forward_noalloc: the problem needs " + std::to_string(n_int32 * sizeof(int32_t)) +
                                " bytes of workspace, the static array holds " + std::to_string(STATIC_SCRATCH_BYTES - STATIC_TABLE_BYTES));
            d_ws = (int32_t *)(static_base + STATIC_TABLE_BYTES);
            return INTATTN_OK;
        }
        const int r = ensure_workspace(ctx, n_int32);
        d_ws = ctx->d_ws;
        return r;
    };
    // the table the kernels read: the context's copy is uploaded only when it differs from what it holds
    // (calls on a context are ordered by the caller); the static array is shared by every context on the
    // GPU, so its table is written on every call
    auto put_table = [&](const std::vector<HeadParams> &tab) -> int {
        if (rm.no_alloc) return upload(ctx, d_hp, tab.data(), tab.size() * sizeof(HeadParams), st, "hipMemcpyAsync(head params)");
        const bool same = ctx->hp_host.size() == tab.size() &&
                          std::memcmp(ctx->hp_host.data(), tab.data(), tab.size() * sizeof(HeadParams)) == 0;
        if (same) return INTATTN_OK;
        const int r = upload(ctx, d_hp, tab.data(), tab.size() * sizeof(HeadParams), st, "hipMemcpyAsync(head params)");
        if (r == INTATTN_OK) ctx->hp_host = tab;
        else ctx->hp_host.clear();
        return r;
    };

    FwdParams p;
    std::memset(&p, 0, sizeof(p));
    p.q = a->q; p.k = a->k; p.v = a->v; p.out = a->out;
    for (int i = 0; i < 3; ++i) {
        p.qs[i] = a->q_stride[i]; p.ks[i] = a->k_stride[i];
        p.vs[i] = a->v_stride[i]; p.os[i] = a->out_stride[i];
    }
    p.B = a->B; p.Hq = a->Hq; p.Hkv = a->Hkv; p.L = a->L;
    p.Lk = a->Lkv ? a->Lkv : a->L;
    p.row_lo = a->causal ? p.Lk - p.L : 0;
    if (comparator && p.Lk != p.L) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "the comparator covers L == Lkv only");
    p.causal = a->causal;
    p.group = a->Hq / a->Hkv;
    p.top = (1 << ctx->lut_bits) - 1;
    int variant = fwd_choose_variant(ctx->variant, a->B, a->Hq, a->L, p.Lk, a->d, a->causal);
    if (variant == 5 && ctx->lut_bits > 5) variant = 4; // the pipelined sweep C holds 32-entry tables; same tiling otherwise
    if (a->scale_mode == 3) variant = 1;                // groups over the key axis: the single-launch kernel
    if (variant == 3 && a->scale_mode == 2) variant = 1; // the split-key single launch takes per-tensor / per-head parameters
    const int rows_per_block = comparator ? 128 : fwd_rows_per_block(variant);
    p.n_qtiles = fwd_row_tiles(p.row_lo, p.L, rows_per_block);
    p.n_chunks = (p.Lk + rows_per_block - 1) / rows_per_block;
    std::memcpy(p.lut, ctx->lut, 64);
    p.dbg_row_max = a->dbg_row_max; p.dbg_row_sum = a->dbg_row_sum; p.dbg_acc = a->dbg_acc;

    // Few query rows against many keys: the split-key kernels (all query heads of a KV head, times
    // the query rows, packed into one MFMA operand of at most 31 rows).
    const int64_t packed_rows = (int64_t)p.group * p.L;
    const bool decode_ok = !comparator && stage == 0 && a->scale_mode < 2 && packed_rows <= 31 && (int64_t)a->B * a->Hkv <= 65535;
    const bool decode = decode_ok && (ctx->variant == 9 || ctx->variant == 10 || (ctx->variant == 0 && p.Lk >= 1024));

    if (dynamic) {
        if (rm.no_alloc) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "intattn_forward_noalloc takes host scales");
        rc = get_tables(a->Hq);
        if (rc) return rc;
        if (a->Hq > ctx->status_cap) {
            int32_t *stw = nullptr;
            const hipError_t e = hipMalloc((void **)&stw, sizeof(int32_t) * (size_t)a->Hq);
            if (e != hipSuccess) return fail(ctx, INTATTN_ERR_NOMEM, std::string("hipMalloc of the status words: ") + hipGetErrorString(e));
            if (ctx->d_status) (void)hipFree(ctx->d_status);
            ctx->d_status = stw;
            ctx->status_cap = a->Hq;
        }
        DeriveParams dp;
        std::memset(&dp, 0, sizeof(dp));
        dp.scale_q = a->scale_q; dp.scale_k = a->scale_k; dp.scale_v = a->scale_v; dp.scale_out = a->scale_out;
        dp.per_head = a->scale_mode != 0;
        dp.Hq = a->Hq;
        dp.group = p.group;
        dp.top = p.top;
        dp.clip = ctx->clip;
        dp.sqrt_d = std::sqrt((double)a->d);
        dp.hp_table = d_hp;
        dp.status = ctx->d_status;
        if (a->scale_mode >= 2) {
            dp.n_rowblk = (a->L + a->q_block - 1) / a->q_block;
            dp.n_entries = (int64_t)a->B * a->Hq * dp.n_rowblk;
            if ((size_t)dp.n_entries > ctx->rowtab_cap) {
                HeadParams *t = nullptr;
                const hipError_t e = hipMalloc((void **)&t, sizeof(HeadParams) * (size_t)dp.n_entries);
                if (e != hipSuccess) return fail(ctx, INTATTN_ERR_NOMEM, std::string("hipMalloc of the row-group table: ") + hipGetErrorString(e));
                if (ctx->d_rowtab) (void)hipFree(ctx->d_rowtab); // waits for work that may still read it
                ctx->d_rowtab = t;
                ctx->rowtab_cap = (size_t)dp.n_entries;
            }
        }
        if (!rm.reserve) {
            ctx->status_n = a->Hq;
            ctx->hp_host.clear(); // the table no longer holds what the host last sent
            if (a->scale_mode >= 2) {
                dp.row_table = ctx->d_rowtab;
                if (a->scale_mode == 3) {
                    dp.Hkv = a->Hkv;
                    dp.n_kblk = (p.Lk + a->k_block - 1) / a->k_block;
                    dp.n_kentries = (int64_t)a->B * a->Hkv * dp.n_kblk;
                }
                const int e = a->scale_mode == 3 ? launch_derive_groups(dp, stream) : launch_derive_rows(dp, stream);
                if (e != 0) return hip_fail(ctx, (hipError_t)e, "launch(derive row-group parameters)");
                p.row_table = ctx->d_rowtab;
                p.q_block = a->q_block;
                p.n_rowblk = dp.n_rowblk;
                p.hp_table = nullptr; // the kernels take every parameter from the row table
                if (a->scale_mode == 3) {
                    p.sq_rows = a->scale_q;
                    p.sk_blocks = a->scale_k;
                    p.k_block = a->k_block;
                    p.n_kblk = dp.n_kblk;
                    p.clip = ctx->clip;
                    p.sqrt_d = dp.sqrt_d;
                    p.head_status = ctx->d_status;
                }
            } else {
                if (stage != 2) { // stage 2 reads what stage 1 derived
                    const int e = launch_derive(dp, stream);
                    if (e != 0) return hip_fail(ctx, (hipError_t)e, "launch(derive head parameters)");
                }
                p.hp_table = d_hp;
            }
        }
    } else if (decode) {
        // every head's parameters in the device table, each with the scheme of its index map
        rc = get_tables(a->Hq);
        if (rc) return rc;
        if (!rm.reserve) {
            std::vector<HeadParams> tab((size_t)a->Hq);
            for (int h = 0; h < a->Hq; ++h) {
                tab[(size_t)h] = dv.hp[a->scale_mode ? (size_t)h : 0];
                tab[(size_t)h].pad[0] = dv.idx_mode;
            }
            rc = put_table(tab);
            if (rc) return rc;
            p.hp_table = d_hp;
        }
    } else if (a->scale_mode == 0) {
        if (!rm.reserve) {
            p.hp_table = nullptr;
            p.hp0 = dv.hp[0];
            p.alpha0 = dv.alpha[0];
            p.sv_over_so0 = dv.svso[0];
        }
    } else {
        // (twice the heads: a second table for sweep C may follow the first)
        rc = get_tables(rm.no_alloc ? a->Hq : 2 * a->Hq);
        if (rc) return rc;
        if (!rm.reserve) {
            if (!dv.hp_c.empty() && !rm.no_alloc && !comparator) {
                std::vector<HeadParams> both(dv.hp);
                both.insert(both.end(), dv.hp_c.begin(), dv.hp_c.end());
                rc = put_table(both);
                p.hp_table_c = d_hp + a->Hq;
            } else {
                rc = put_table(dv.hp);
            }
            if (rc) return rc;
            if (comparator && !(ctx->alpha_host == dv.alpha && ctx->svso_host == dv.svso)) {
                const size_t n = (size_t)a->Hq;
                rc = upload(ctx, ctx->d_alpha, dv.alpha.data(), n * sizeof(float), st, "hipMemcpyAsync(comparator scales)");
                if (rc == INTATTN_OK) rc = upload(ctx, ctx->d_svso, dv.svso.data(), n * sizeof(float), st, "hipMemcpyAsync(comparator scales)");
                if (rc) return rc;
                ctx->alpha_host = dv.alpha;
                ctx->svso_host = dv.svso;
            }
            p.hp_table = d_hp;
            p.alpha_table = ctx->d_alpha;
            p.svso_table = ctx->d_svso;
        }
    }

    if (decode) {
        const size_t groups = (size_t)a->B * a->Hkv, R = (size_t)packed_rows;
        const size_t nt32 = 4 * (((size_t)p.Lk + 127) / 128);
        // tiles per workgroup: as many as leave about a thousand workgroups (four per compute unit: all of
        // them resident at once, so no second, partly filled round of workgroups; five per unit measured
        // slower), at most 64
        const size_t tiles = groups * (nt32 / 4);
        size_t tpw = tiles / 1024 < 1 ? 1 : (tiles / 1024 > 64 ? 64 : tiles / 1024);
        // One launch, with the scores of a chunk held in LDS: as 16-bit distances where every clip threshold fits
        // 16 bits and is known here (host scales; chunks of at most 64 / R tiles), else as raw 32-bit scores
        // (chunks of at most 32 / R tiles).  Callers that may not allocate and variant 10 take the separate
        // launches, which pass 32-bit scores through the workspace.
        const bool fused = !rm.no_alloc && ctx->variant != 10;
        bool wide = dynamic;
        if (fused && !dynamic && !rm.reserve)
            for (const HeadParams &h : dv.hp) wide = wide || h.c_int > 65535;
        if (fused && tpw > (wide ? 32 : 64) / R) tpw = (wide ? 32 : 64) / R;
        const size_t chunks = (nt32 / 4 + tpw - 1) / tpw;
        const size_t n_scores = groups * nt32 * 2 * R * 16, n_idx = groups * nt32 * 2 * R * 4, n_part = groups * chunks * 4 * R;
        const size_t n_acc = groups * chunks * R * (size_t)a->d;
        rc = get_ws(fused && !rm.reserve ? n_acc : n_scores + n_idx + 2 * n_part + n_acc);
        if (rc) return rc;
        if (fused && groups > ctx->dec_state_groups) {
            uint32_t *stt = nullptr;
            hipError_t e = hipMalloc((void **)&stt, groups * DEC_STATE_WORDS * sizeof(uint32_t));
            if (e == hipSuccess && (e = hipMemset(stt, 0, groups * DEC_STATE_WORDS * sizeof(uint32_t))) != hipSuccess) (void)hipFree(stt);
            if (e != hipSuccess) return fail(ctx, INTATTN_ERR_NOMEM, std::string("hipMalloc of the split-key group state: ") + hipGetErrorString(e));
            if (ctx->d_dec_state) (void)hipFree(ctx->d_dec_state); // waits for work that may still use it
            ctx->d_dec_state = stt;
            ctx->dec_state_groups = groups;
        } else if (fused && rm.reserve) {
            // a launch that gave up waiting leaves counters behind: reserving again starts from zero
            const hipError_t e = hipMemset(ctx->d_dec_state, 0, ctx->dec_state_groups * DEC_STATE_WORDS * sizeof(uint32_t));
            if (e != hipSuccess) return hip_fail(ctx, e, "hipMemset(split-key group state)");
        }
        if (rm.reserve) return INTATTN_OK;
        p.dec_rows = (int32_t)R;
        p.dec_nt32 = (int32_t)nt32;
        p.dec_tpw = (int32_t)tpw;
        p.dec_np = (int32_t)(chunks * 4);
        if (fused) {
            p.dec_acc = d_ws;
            p.dec_state = ctx->d_dec_state;
            p.dec_spin_limit = 1 << 22;
            p.dec_wide = wide ? 1 : 0;
            // testing aid: a smaller bound makes the workgroups give up, which the tests of that path need
            if (const char *lim = std::getenv("INTATTN_SPLITKEY_SPIN_LIMIT")) {
                const long v = std::strtol(lim, nullptr, 10);
                p.dec_spin_limit = v < 0 ? 0 : (v > (1 << 22) ? (1 << 22) : (int32_t)v);
            }
        } else {
            p.dec_scores = d_ws; // every part is a multiple of 4 words: 16-byte alignment holds
            p.dec_idx = p.dec_scores + n_scores;
            p.dec_acc = p.dec_idx + n_idx;
            p.dec_pmax = p.dec_acc + n_acc;
            p.dec_psum = p.dec_pmax + n_part;
        }
        const int herr = launch_decode(p, a->d, stream);
        if (herr != 0) return hip_fail(ctx, (hipError_t)herr, "launch(split-key forward)");
        ctx->err.clear();
        return INTATTN_OK;
    }
    if (!comparator && variant != 3) { // (the split-key single launch passes nothing through memory)
        const size_t rows = (size_t)a->B * a->Hq * a->L;
        const size_t cs = (size_t)a->B * a->Hkv * p.n_chunks * a->d;
        rc = get_ws(2 * rows + cs);
        if (rc) return rc;
        p.ws_row_max = d_ws;
        p.ws_row_sum = p.ws_row_max + rows;
        p.ws_colsum = p.ws_row_sum + rows;
    }
    if (rm.reserve) return INTATTN_OK;

    const int herr = comparator ? launch_quantonly(p, a->d, ctx->variant, stream)
                                : launch_fwd(p, a->d, dv.idx_mode, variant, stage, stream);
    if (herr == (int)hipErrorNotSupported)
        return fail(ctx, INTATTN_ERR_UNSUPPORTED, "the kernel variant in use for this problem is a single launch: no stages");
    if (herr != 0) return hip_fail(ctx, (hipError_t)herr, comparator ? "launch(quant-only)" : "launch(intattn forward)");
    ctx->err.clear();
    return INTATTN_OK;
}

} // namespace

extern "C" {

int intattn_create(intattn_ctx **out, const intattn_config *cfg)
{
    if (!out || !cfg) return fail(nullptr, INTATTN_ERR_INVALID_ARG, "out and cfg must be non-NULL");
    *out = nullptr;
    if (cfg->lut_bits < 1 || cfg->lut_bits > 6) return fail(nullptr, INTATTN_ERR_UNSUPPORTED, "lut_bits must be in 1..6");
    if (!(cfg->clip > 0.0) || !std::isfinite(cfg->clip)) return fail(nullptr, INTATTN_ERR_INVALID_ARG, "clip must be finite and > 0");
    if (!fwd_variant_known(cfg->variant)) return fail(nullptr, INTATTN_ERR_INVALID_ARG, "unknown kernel variant");
    if (cfg->reserved != 0) return fail(nullptr, INTATTN_ERR_INVALID_ARG, "reserved must be 0");
    if (cfg->device < -1) return fail(nullptr, INTATTN_ERR_INVALID_ARG, "no such HIP device");
    if (cfg->device >= 0) {
        int ndev = 0;
        hipError_t e = hipGetDeviceCount(&ndev);
        if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDeviceCount");
        if (cfg->device >= ndev) return fail(nullptr, INTATTN_ERR_INVALID_ARG, "no such HIP device");
    }
    intattn_ctx *ctx = new (std::nothrow) intattn_ctx();
    if (!ctx) return fail(nullptr, INTATTN_ERR_NOMEM, "out of host memory");
    ctx->device = cfg->device;
    ctx->lut_bits = cfg->lut_bits;
    ctx->clip = cfg->clip;
    ctx->variant = cfg->variant;
    // Eq. lut_re and Eq. lut16
    const int n = 1 << cfg->lut_bits;
    for (int i = 0; i < n - 1; ++i)
        ctx->lut[i] = (uint8_t)std::floor(255.0 * std::exp(-cfg->clip * (double)i / (double)(n - 1)) + 0.5);
    ctx->lut[n - 1] = 0;
    if (ctx->device >= 0) {
        DeviceGuard guard(ctx->device);
        hipError_t e = guard.status;
        // pinned staging for table uploads
        for (Staging &sg : ctx->stage) {
            if (e == hipSuccess) e = hipHostMalloc((void **)&sg.host, STAGING_BYTES, hipHostMallocDefault);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&sg.done, hipEventDisableTiming);
        }
        // this GPU's copy of the static workspace of intattn_forward_noalloc
        if (e == hipSuccess && ctx->device < MAX_DEVICES) {
            std::lock_guard<std::mutex> lock(g_scratch_mu);
            if (!g_scratch_ptr[ctx->device]) {
                void *ptr = nullptr;
                e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
                if (e == hipSuccess) g_scratch_ptr[ctx->device] = ptr;
            }
        }
        if (e != hipSuccess) {
            const int rc = hip_fail(nullptr, e, "intattn_create (staging buffers / static workspace)");
            intattn_destroy(ctx);
            return rc;
        }
    }
    *out = ctx;
    return INTATTN_OK;
}

int intattn_forward(intattn_ctx *ctx, const intattn_args *args, void *hip_stream)
{
    return run(ctx, args, hip_stream, RunMode{});
}

int intattn_forward_noalloc(intattn_ctx *ctx, const intattn_args *args, void *hip_stream)
{
    RunMode rm;
    rm.no_alloc = true;
    return run(ctx, args, hip_stream, rm);
}

int intattn_reserve(intattn_ctx *ctx, const intattn_args *args, int32_t dynamic)
{
    RunMode rm;
    rm.reserve = true;
    rm.dynamic = dynamic != 0;
    return run(ctx, args, nullptr, rm);
}

int intattn_forward_stage(intattn_ctx *ctx, const intattn_args *args, void *hip_stream, int32_t stage)
{
    if (stage < 0 || stage > 2) return fail(ctx, INTATTN_ERR_INVALID_ARG, "stage must be 0, 1 or 2");
    RunMode rm;
    rm.stage = stage;
    return run(ctx, args, hip_stream, rm);
}

int intattn_forward_dynamic(intattn_ctx *ctx, const intattn_args *args, void *hip_stream)
{
    RunMode rm;
    rm.dynamic = true;
    return run(ctx, args, hip_stream, rm);
}

int intattn_dynamic_status(intattn_ctx *ctx, int32_t *status)
{
    if (!ctx) return INTATTN_ERR_INVALID_ARG;
    if (!status) return fail(ctx, INTATTN_ERR_INVALID_ARG, "status is NULL");
    *status = 0;
    if (!ctx->d_status || ctx->status_n < 1) return INTATTN_OK; // no dynamic call yet
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return hip_fail(ctx, guard.status, "hipSetDevice");
    std::vector<int32_t> words((size_t)ctx->status_n, 0);
    const hipError_t e = hipMemcpy(words.data(), ctx->d_status, sizeof(int32_t) * words.size(), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipMemcpy(status)");
    for (int32_t w : words)
        if (w != 0) *status = 1;
    return INTATTN_OK;
}

int intattn_index_softmax(intattn_ctx *ctx, const intattn_softmax_args *a, void *hip_stream)
{
    if (!ctx) return INTATTN_ERR_INVALID_ARG;
    if (!a) return fail(ctx, INTATTN_ERR_INVALID_ARG, "args is NULL");
    if (ctx->device < 0) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "host-only context: no device to run on");
    if (a->rows < 1 || a->cols < 1) return fail(ctx, INTATTN_ERR_INVALID_ARG, "rows and cols must be >= 1");
    if (a->cols > (1 << 29)) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "cols must not exceed 2^29");
    if (a->c_int < 1 || a->c_int > (1 << 30)) return fail(ctx, INTATTN_ERR_INVALID_ARG, "c_int must be in 1 .. 2^30");
    if (!a->logits || !a->prob) return fail(ctx, INTATTN_ERR_INVALID_ARG, "logits and prob must be non-NULL");
    if ((const void *)a->prob == (const void *)a->logits) return fail(ctx, INTATTN_ERR_INVALID_ARG, "prob must not alias logits");
    if (((uintptr_t)a->logits) & 3u) return fail(ctx, INTATTN_ERR_INVALID_ARG, "logits must be 4-byte aligned");
    if (a->logits_stride < 4 * (int64_t)a->cols || (a->logits_stride & 3) != 0)
        return fail(ctx, INTATTN_ERR_INVALID_ARG, "logits_stride must be a multiple of 4 and at least 4 * cols");
    if (a->prob_stride < (int64_t)a->cols) return fail(ctx, INTATTN_ERR_INVALID_ARG, "prob_stride must be at least cols");
    if (a->causal != 0 && a->causal != 1) return fail(ctx, INTATTN_ERR_INVALID_ARG, "causal must be 0 or 1");
    if (a->causal && (a->rows_per_matrix < 1 || a->rows_per_matrix > a->cols || a->rows % a->rows_per_matrix != 0))
        return fail(ctx, INTATTN_ERR_INVALID_ARG, "rows_per_matrix must be in 1 .. cols and divide rows");
    const int64_t blocks = a->cols <= 2048 ? (a->rows + 3) / 4 : a->rows;
    if (blocks > 2147483647LL) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "problem needs more than 2^31-1 workgroups");
    SoftmaxParams p;
    std::memset(&p, 0, sizeof(p));
    p.logits = a->logits; p.prob = a->prob;
    p.ls = a->logits_stride; p.ps = a->prob_stride;
    p.rows = a->rows; p.cols = a->cols;
    p.vec_in = ((((uintptr_t)a->logits) & 15u) == 0 && (a->logits_stride & 15) == 0) ? 1 : 0;
    p.vec_out = ((((uintptr_t)a->prob) & 3u) == 0 && (a->prob_stride & 3) == 0) ? 1 : 0;
    p.rows_per_matrix = a->causal ? a->rows_per_matrix : 1;
    p.causal = a->causal;
    p.top = (1 << ctx->lut_bits) - 1;
    std::memcpy(p.lut, ctx->lut, 64);
    // the cheapest exact index map for this threshold
    p.hp.c_int = a->c_int;
    if (find_top24((uint32_t)a->c_int, (uint32_t)p.top, &p.hp)) p.hp.pad[0] = IDX_TOP24;
    else if (find_fp64((uint32_t)a->c_int, (uint32_t)p.top, &p.hp)) p.hp.pad[0] = IDX_FP64;
    else return fail(ctx, INTATTN_ERR_UNSUPPORTED, "no exact index map for this c_int");
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return hip_fail(ctx, guard.status, "hipSetDevice");
    const int herr = launch_index_softmax(p, hip_stream);
    if (herr != 0) return hip_fail(ctx, (hipError_t)herr, "launch(index softmax)");
    ctx->err.clear();
    return INTATTN_OK;
}

int intattn_quantize_batch(intattn_ctx *ctx, const intattn_quant_args *args, int32_t count, void *hip_stream)
{
    if (!ctx) return INTATTN_ERR_INVALID_ARG;
    if (!args) return fail(ctx, INTATTN_ERR_INVALID_ARG, "args is NULL");
    if (count < 1 || count > 4) return fail(ctx, INTATTN_ERR_INVALID_ARG, "count must be in 1..4");
    if (ctx->device < 0) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "host-only context: no device to run on");
    QuantParams ps[4];
    int64_t groups[4], total = 0;
    for (int t = 0; t < count; ++t) {
        const intattn_quant_args *a = args + t;
        if (a->B < 1 || a->H < 1 || a->L < 1 || a->d < 8) return fail(ctx, INTATTN_ERR_INVALID_ARG, "B, H, L must be >= 1 and d >= 8");
        if (a->d % 8 != 0) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "d must be a multiple of 8");
        if ((int64_t)a->B * a->H > 65535) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "B * H must not exceed 65535");
        if ((int64_t)a->L * (a->d / 8) > 2147483647LL) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "L * d / 8 must fit 31 bits");
        if (a->dtype < 0 || a->dtype > 2) return fail(ctx, INTATTN_ERR_INVALID_ARG, "dtype must be 0 (fp32), 1 (fp16) or 2 (bf16)");
        if (a->scale_mode < 0 || a->scale_mode > 2) return fail(ctx, INTATTN_ERR_INVALID_ARG, "scale_mode must be 0, 1 or 2");
        if (a->scale_mode == 2 && a->q_block < 1) return fail(ctx, INTATTN_ERR_INVALID_ARG, "scale_mode 2 needs q_block >= 1");
        if (a->scale_mode == 2 && count != 1)
            return fail(ctx, INTATTN_ERR_UNSUPPORTED, "scale_mode 2 (a scale per block of rows) takes one tensor per call");
        if (a->reserved != 0) return fail(ctx, INTATTN_ERR_INVALID_ARG, "reserved must be 0");
        if (a->scale_mode == 2 && (int64_t)a->B * a->H * ((a->L + a->q_block - 1) / a->q_block) > 2147483647LL)
            return fail(ctx, INTATTN_ERR_UNSUPPORTED, "more than 2^31-1 groups");
        if (!a->src || !a->dst || !a->scales) return fail(ctx, INTATTN_ERR_INVALID_ARG, "src, dst, scales must be non-NULL");
        if ((const void *)a->dst == a->src) return fail(ctx, INTATTN_ERR_INVALID_ARG, "dst must not alias src");
        if ((((uintptr_t)a->src) & 15u) || (((uintptr_t)a->dst) & 7u))
            return fail(ctx, INTATTN_ERR_INVALID_ARG, "src must be 16-byte aligned and dst 8-byte aligned");
        const int64_t es = a->dtype == 0 ? 4 : 2;
        for (int i = 0; i < 3; ++i) {
            if (a->src_stride[i] < 0 || a->dst_stride[i] < 0 || (a->src_stride[i] & 15) != 0 || (a->dst_stride[i] & 7) != 0)
                return fail(ctx, INTATTN_ERR_INVALID_ARG, "src strides must be non-negative multiples of 16, dst strides of 8");
        }
        if (a->src_stride[2] < es * a->d || a->dst_stride[2] < a->d)
            return fail(ctx, INTATTN_ERR_INVALID_ARG, "the L strides must cover a row of d elements");
        QuantParams &p = ps[t];
        std::memset(&p, 0, sizeof(p));
        p.src = a->src; p.dst = a->dst;
        for (int i = 0; i < 3; ++i) { p.ss[i] = a->src_stride[i]; p.ds[i] = a->dst_stride[i]; }
        p.B = a->B; p.H = a->H; p.L = a->L; p.d = a->d;
        p.dtype = a->dtype; p.per_head = a->scale_mode;
        p.q_block = a->q_block;
        p.scales = a->scales;
        p.n_partial = quantize_partials_per_slice(a->B, a->H, a->L, a->d);
        groups[t] = (int64_t)a->B * a->H * p.n_partial;
        total += groups[t];
    }
    if (total > 2147483647LL) return fail(ctx, INTATTN_ERR_UNSUPPORTED, "the batch needs more than 2^31-1 workgroups");
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return hip_fail(ctx, guard.status, "hipSetDevice");
    if (total > ctx->amax_cap) {
        float *m = nullptr;
        const hipError_t e = hipMalloc((void **)&m, sizeof(float) * (size_t)total);
        if (e != hipSuccess) return fail(ctx, INTATTN_ERR_NOMEM, std::string("hipMalloc of the quantizer scratch: ") + hipGetErrorString(e));
        if (ctx->d_amax) (void)hipFree(ctx->d_amax);
        ctx->d_amax = m;
        ctx->amax_cap = total;
    }
    int64_t off = 0;
    for (int t = 0; t < count; ++t) {
        ps[t].partial = ctx->d_amax + off; // each tensor's partial maxima
        off += groups[t];
    }
    const int herr = launch_quantize(ps, count, hip_stream);
    if (herr != 0) return hip_fail(ctx, (hipError_t)herr, "launch(quantize)");
    ctx->err.clear();
    return INTATTN_OK;
}

int intattn_quantize(intattn_ctx *ctx, const intattn_quant_args *a, void *hip_stream)
{
    return intattn_quantize_batch(ctx, a, 1, hip_stream);
}

int intattn_forward_quantonly(intattn_ctx *ctx, const intattn_args *args, void *hip_stream)
{
    RunMode rm;
    rm.comparator = true;
    return run(ctx, args, hip_stream, rm);
}

int intattn_derive_params(const intattn_ctx *ctx, float s_q, float s_k, float s_v, float s_o, int32_t d,
                          int64_t *c_int, int32_t *rq_mult, int32_t *rq_shift)
{
    if (!ctx || d < 1) return INTATTN_ERR_INVALID_ARG;
    if (!good_scale(s_q) || !good_scale(s_k) || !good_scale(s_v) || !good_scale(s_o)) return INTATTN_ERR_INVALID_ARG;
    int32_t m = 0, sh = 0;
    if (!derive_requant(s_v, s_o, &m, &sh)) return INTATTN_ERR_INVALID_ARG;
    if (c_int) *c_int = derive_c_int(ctx->clip, s_q, s_k, d);
    if (rq_mult) *rq_mult = m;
    if (rq_shift) *rq_shift = sh;
    return INTATTN_OK;
}

int intattn_derive_index_map(const intattn_ctx *ctx, int64_t c_int, int32_t *mode, uint32_t *mul, uint32_t *add,
                             int32_t *shift)
{
    if (!ctx || c_int < 1 || c_int > 1073741824LL || !mode || !mul || !add || !shift) return INTATTN_ERR_INVALID_ARG;
    HeadParams hp{};
    const uint32_t top = (1u << ctx->lut_bits) - 1u;
    if (*mode == IDX_MAD24) {
        *mode = find_mad24((uint32_t)c_int, top, &hp) ? IDX_MAD24 : IDX_FP64;
    } else if (*mode == IDX_FP32) {
        *mode = find_fp32((uint32_t)c_int, top, &hp) ? IDX_FP32 : IDX_FP64;
    } else if (*mode == IDX_MULHI24) {
        *mode = find_mulhi24((uint32_t)c_int, top, &hp) ? IDX_MULHI24 : IDX_FP64;
    } else if (*mode == IDX_TOP24) {
        *mode = find_top24((uint32_t)c_int, top, &hp) ? IDX_TOP24 : IDX_FP64;
    } else {
        *mode = IDX_FP64;
    }
    if (*mode == IDX_FP64) {
        if (!find_fp64((uint32_t)c_int, top, &hp)) return INTATTN_ERR_UNSUPPORTED;
        *mul = hp.idx_mul; // bits of +r: low word, high word
        *add = hp.idx_add ^ 0x80000000u;
        *shift = 0;
        return INTATTN_OK;
    }
    // report the mathematical constants (the kernel-side fields hold them negated)
    if (*mode == IDX_FP32) {
        *mul = hp.idx_mul ^ 0x80000000u; // bits of +r
        *add = 0;
        *shift = 0;
        return INTATTN_OK;
    }
    *mul = (uint32_t)(-(int32_t)hp.idx_mul);
    *add = *mode == IDX_MULHI24 ? (uint32_t)(-(int32_t)hp.idx_add) : hp.idx_add;
    *shift = hp.idx_shift;
    return INTATTN_OK;
}

int intattn_get_lut(const intattn_ctx *ctx, uint8_t *dst, int32_t cap)
{
    if (!ctx || !dst) return INTATTN_ERR_INVALID_ARG;
    const int n = 1 << ctx->lut_bits;
    if (cap < n) return INTATTN_ERR_INVALID_ARG;
    std::memcpy(dst, ctx->lut, (size_t)n);
    return n;
}

const char *intattn_last_error(const intattn_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

void intattn_destroy(intattn_ctx *ctx)
{
    if (!ctx) return;
    if (ctx->device >= 0) {
        DeviceGuard guard(ctx->device);
        if (ctx->d_hp) (void)hipFree(ctx->d_hp);
        if (ctx->d_alpha) (void)hipFree(ctx->d_alpha);
        if (ctx->d_svso) (void)hipFree(ctx->d_svso);
        if (ctx->d_ws) (void)hipFree(ctx->d_ws);
        if (ctx->d_amax) (void)hipFree(ctx->d_amax);
        if (ctx->d_status) (void)hipFree(ctx->d_status);
        if (ctx->d_rowtab) (void)hipFree(ctx->d_rowtab);
        if (ctx->d_dec_state) (void)hipFree(ctx->d_dec_state);
        for (Staging &sg : ctx->stage) {
            if (sg.pending) (void)hipEventSynchronize(sg.done);
            if (sg.done) (void)hipEventDestroy(sg.done);
            if (sg.host) (void)hipHostFree(sg.host);
        }
    }
    delete ctx;
}

} // extern "C"
