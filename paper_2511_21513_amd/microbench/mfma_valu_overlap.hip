// Microbenchmark behind the cycle model of the attention kernels on gfx950: does v_mfma_i32_32x32x32_i8 of one wave
// overlap with vector instructions of another wave on the same SIMD?  The instruction mix is that of sweep C (per
// 32 x 32 block of scores: a chain of four MFMAs for the scores, four for P.V, and per score a clip, a 24-bit
// multiply-add and a byte permute that read the MFMA results and feed the next MFMA operand).  Every kernel computes a
// defined result (written out as a checksum); nothing is removed to time it.  One workgroup per compute unit:
// 256 threads = one wave per SIMD, 512 threads = two waves per SIMD.
//   interleaved: one MFMA, then an eighth of the vector work, eight times (the software pipeline of sweep C)
//   bursts:      eight MFMAs, then all the vector work (the phase-ordered kernels)
//   ping-pong:   bursts, the two waves of a SIMD held in opposite phases by a barrier between phases
//                (with and without raised priority in the MFMA burst)
//   MFMA only / vector only: the two parts alone;  split: one wave of a SIMD issues only the MFMAs of two
//                iterations, the other only the vector work of two iterations (no dependence between them)
// Build and run:  hipcc -O3 --offload-arch=gfx950 -mllvm -amdgpu-mfma-vgpr-form=1 -o /tmp/overlap mfma_valu_overlap.hip && /tmp/overlap
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

// MODE 0: 8 x (1 MFMA + NV/8 vector ops) interleaved; 1: burst of 8 MFMAs then NV vector ops; 2: bursts with the two
// halves of the workgroup in opposite phases, a barrier between phases; 3: as 2 with raised priority in the MFMA burst.
template <int MODE, int NV>
__global__ __launch_bounds__(512) void k(int iters, int *out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool groupB = (blockDim.x == 512) && wave >= 4;
    v16i s, o0, o1, o2, o3;
    for (int i = 0; i < 16; ++i) s[i] = o0[i] = o1[i] = o2[i] = o3[i] = 0;
    v4i qf[4], kf[4], vf[4], pf = {1, 2, 3, 4};
    for (int j = 0; j < 4; ++j) { qf[j] = v4i{lane, 1, 2, 3 + j}; kf[j] = v4i{1, lane & 3, 2, j}; vf[j] = v4i{j, 2, lane & 7, 1}; }
    const int bound = -5, mul = 77, addc = 12345;
    auto mfma_burst = [&]() __attribute__((always_inline)) {
        if (MODE == 3) __builtin_amdgcn_s_setprio(3);
        s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[0], qf[0], v16i{0,0,0,0,0,0,0,0,0,0,0,0,0,0,0,0}, 0, 0, 0);
        s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[1], qf[1], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[2], qf[2], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[3], qf[3], s, 0, 0, 0);
        o0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[0], pf, o0, 0, 0, 0);
        o1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[1], pf, o1, 0, 0, 0);
        o2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[2], pf, o2, 0, 0, 0);
        o3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[3], pf, o3, 0, 0, 0);
        if (MODE == 3) __builtin_amdgcn_s_setprio(0);
    };
    // NV vector instructions on the scores: per score max + mad24 (+ a permute every second score), results into pf
    auto valu_burst = [&]() __attribute__((always_inline)) {
        int acc[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < NV / 3; ++e) {
            int c, r, t;
            asm volatile("v_max_i32 %0, %1, %2" : "=v"(c) : "v"(s[e % 16]), "v"(bound + e));
            asm volatile("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(c), "v"(mul), "v"(addc));
            asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(t) : "v"(r), "v"(acc[e % 4]), "v"(0x07020100 + (e & 1)));
            acc[e % 4] = t;
        }
        pf = v4i{acc[0] & 0x01010101, acc[1] & 0x01010101, acc[2] & 0x01010101, acc[3] & 0x01010101};
    };
    for (int it = 0; it < iters; ++it) {
        if (MODE == 0) {
            // fine interleave: one MFMA, then an eighth of the vector work (on the previous scores)
            int acc[4] = {0, 0, 0, 0};
            v16i sp = s;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) {
                if (sl == 0) s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[0], qf[0], v16i{0,0,0,0,0,0,0,0,0,0,0,0,0,0,0,0}, 0, 0, 0);
                else if (sl < 4) s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[sl], qf[sl], s, 0, 0, 0);
                else if (sl == 4) o0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[0], pf, o0, 0, 0, 0);
                else if (sl == 5) o1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[1], pf, o1, 0, 0, 0);
                else if (sl == 6) o2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[2], pf, o2, 0, 0, 0);
                else o3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[3], pf, o3, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = sl * (NV / 24); e < (sl + 1) * (NV / 24); ++e) {
                    int c, r, t;
                    asm volatile("v_max_i32 %0, %1, %2" : "=v"(c) : "v"(sp[e % 16]), "v"(bound + e));
                    asm volatile("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(c), "v"(mul), "v"(addc));
                    asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(t) : "v"(r), "v"(acc[e % 4]), "v"(0x07020100 + (e & 1)));
                    acc[e % 4] = t;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            pf = v4i{acc[0] & 0x01010101, acc[1] & 0x01010101, acc[2] & 0x01010101, acc[3] & 0x01010101};
        } else if (MODE == 4) {
            mfma_burst();
            __builtin_amdgcn_sched_barrier(0);
        } else if (MODE == 5) {
            valu_burst();
            __builtin_amdgcn_sched_barrier(0);
        } else if (MODE == 6) {
            // one wave of a SIMD only issues MFMAs, the other only vector instructions (two iterations' worth each,
            // so that the work per iteration and SIMD equals that of the other modes)
            if (!groupB) { mfma_burst(); __builtin_amdgcn_sched_barrier(0); mfma_burst(); }
            else { valu_burst(); __builtin_amdgcn_sched_barrier(0); valu_burst(); }
            __builtin_amdgcn_sched_barrier(0);
        } else if (MODE == 1) {
            mfma_burst();
            __builtin_amdgcn_sched_barrier(0);
            valu_burst();
            __builtin_amdgcn_sched_barrier(0);
        } else {
            if (!groupB) {
                mfma_burst();
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
                valu_burst();
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
            } else {
                valu_burst();
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
                mfma_burst();
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
            }
        }
    }
    int x = pf[0] ^ pf[1] ^ pf[2] ^ pf[3];
    for (int i = 0; i < 16; ++i) x ^= s[i] ^ o0[i] ^ o1[i] ^ o2[i] ^ o3[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = x;
}

template <int MODE, int NV> int run(const char *name, int threads, int *d_out)
{
    const int iters = 20000, grid = 256;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL((k<MODE, NV>), dim3(grid), dim3(threads), 0, 0, 100, d_out);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL((k<MODE, NV>), dim3(grid), dim3(threads), 0, 0, iters, d_out);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms = 0; CHECK(hipEventElapsedTime(&ms, e0, e1));
    const int waves_per_simd = threads / 256;
    printf("%-34s NV=%3d waves/SIMD=%d  %7.1f ns per iteration per wave-slot, %7.1f ns per block per SIMD\n", name, NV, waves_per_simd,
           ms * 1e6 / iters, ms * 1e6 / iters / waves_per_simd);
    fflush(stdout);
    return 0;
}

int main()
{
    int *d_out; CHECK(hipMalloc(&d_out, 256 * 512 * sizeof(int)));
    if (run<4, 48>("MFMA only", 256, d_out)) return 1;
    if (run<4, 48>("MFMA only", 512, d_out)) return 1;
    if (run<5, 48>("vector only", 256, d_out)) return 1;
    if (run<5, 48>("vector only", 512, d_out)) return 1;
    if (run<5, 96>("vector only", 512, d_out)) return 1;
    if (run<6, 48>("split: MFMA wave + vector wave", 512, d_out)) return 1;
    if (run<6, 96>("split: MFMA wave + vector wave", 512, d_out)) return 1;
    if (run<0, 48>("interleaved", 256, d_out)) return 1;
    if (run<1, 48>("bursts", 256, d_out)) return 1;
    if (run<0, 48>("interleaved", 512, d_out)) return 1;
    if (run<1, 48>("bursts, no sync", 512, d_out)) return 1;
    if (run<2, 48>("bursts, ping-pong barriers", 512, d_out)) return 1;
    if (run<3, 48>("ping-pong + setprio", 512, d_out)) return 1;
    if (run<0, 96>("interleaved", 256, d_out)) return 1;
    if (run<1, 96>("bursts", 256, d_out)) return 1;
    if (run<0, 96>("interleaved", 512, d_out)) return 1;
    if (run<1, 96>("bursts, no sync", 512, d_out)) return 1;
    if (run<2, 96>("bursts, ping-pong barriers", 512, d_out)) return 1;
    if (run<3, 96>("ping-pong + setprio", 512, d_out)) return 1;
    CHECK(hipFree(d_out));
    return 0;
}
