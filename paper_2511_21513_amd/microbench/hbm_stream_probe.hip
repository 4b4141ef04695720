// How fast can this GPU stream a tensor from HBM with the access shape of the split-key kernels, and what does
// a small store per read cost?  A workgroup of four waves walks 16 KiB tiles; wave w takes the 4 KiB piece w of
// every tile (INTER 1) or a contiguous run of its own (INTER 0); a lane reads the 16 bytes of "its" 128-byte row
// that an MFMA operand would hold, DEPTH pieces in flight per wave.  ST 1: eight lanes store 64 bytes each per
// piece (16-byte stores at a stride of 64); ST 2: 32 lanes store 16 bytes each (whole lines).  Successive
// launches read successive 256 MiB regions of a 2 GiB buffer, so nothing is served from the Infinity Cache.
// Every kernel reads what it is timed for and produces a defined result.
//   hipcc -O3 --offload-arch=gfx950 -o /tmp/hbm_stream_probe paper_2511_21513_amd/microbench/hbm_stream_probe.hip && /tmp/hbm_stream_probe
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
typedef int v4i __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

// INTER 1: interleaved (wave w takes piece w of every 16 KiB), 0: each wave a contiguous run
// ST 1: 8 lanes store 64 B each per piece
template <int INTER, int ST, int DEPTH>
__global__ __launch_bounds__(256) void rd(const int8_t *src, int tpw, int32_t *out, int32_t *sink)
{
    const int lane = threadIdx.x & 63, n = lane & 31, h = lane >> 5, w = threadIdx.x >> 6;
    const int8_t *base = src + (int64_t)blockIdx.x * tpw * 16384 + (INTER ? w * 4096 : w * tpw * 4096);
    const int64_t step = INTER ? 16384 : 4096;
    v4i buf[DEPTH][4];
    v4i acc = {0, 0, 0, 0};
    auto load = [&](int s, v4i *b) __attribute__((always_inline)) {
        const int8_t *t = base + (int64_t)(s < tpw ? s : tpw - 1) * step;
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = *(const v4i *)(t + n * 128 + 32 * j + 16 * h);
    };
    auto use = [&](int s, v4i *b) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc ^= b[j];
        if (ST == 2) {
            if (lane < 32) *(v4i *)(out + (((int64_t)blockIdx.x * tpw + s) * 4 + w) * 128 + lane * 4) = acc;
        } else if (ST && n < 4) {
            int32_t *dst = out + (((int64_t)blockIdx.x * tpw + s) * 4 + w) * 128 + (h * 4 + n) * 16;
#pragma unroll
            for (int g = 0; g < 4; ++g) *(v4i *)(dst + 4 * g) = acc;
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load(d, buf[d]);
    int s = 0;
    for (; s + DEPTH - 1 < tpw; s += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            use(s + d, buf[d]);
            load(s + d + DEPTH, buf[d]);
        }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) if (s + d < tpw) use(s + d, buf[d]);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678) sink[0] = 1;
}

template <int INTER, int ST, int DEPTH>
int run(const int8_t *src, int32_t *out, int32_t *sink, int tpw)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int64_t region = 256ll << 20;
    const int wg = (int)(region / (tpw * 16384ll));
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL((rd<INTER, ST, DEPTH>), dim3(wg), dim3(256), 0, 0, src + (i % 8) * region, tpw, out, sink);
    CK(hipEventRecord(e0, 0));
    const int reps = 24;
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL((rd<INTER, ST, DEPTH>), dim3(wg), dim3(256), 0, 0, src + (i % 8) * region, tpw, out, sink);
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    printf("inter %d stores %d depth %d tpw %2d wg %5d: %.1f us  %.0f GB/s read\n", INTER, ST, DEPTH, tpw, wg, ms / reps * 1e3, region / (ms / reps * 1e-3) / 1e9);
    fflush(stdout);
    return 0;
}

int main()
{
    const int64_t bytes = 2048ll << 20;
    int8_t *src; int32_t *out, *sink;
    CK(hipMalloc(&src, bytes)); CK(hipMalloc(&out, 64 << 20)); CK(hipMalloc(&sink, 64));
    CK(hipMemset(src, 1, bytes));
    for (int tpw : {16, 32, 64}) {
        if (run<0, 0, 3>(src, out, sink, tpw)) return 1;
        if (run<1, 0, 3>(src, out, sink, tpw)) return 1;
        if (run<1, 1, 3>(src, out, sink, tpw)) return 1;
        if (run<1, 2, 3>(src, out, sink, tpw)) return 1;
        if (run<1, 0, 6>(src, out, sink, tpw)) return 1;
    }
    return 0;
}
