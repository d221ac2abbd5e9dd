// Stand-alone measurement, not part of the library: the rate of v_mfma_f32_16x16x32_bf16 issued from registers
// only (no memory traffic), i.e. what the matrix units of an MI355X sustain under the instruction mix of the
// prompt projections (Section 3.2: the verification / prompt rows are dense contractions).
// Build and run:  hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -o mfma_rate mfma_rate.hip && ./mfma_rate
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("ERR %s at %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// MODE 0: 32 accumulators, 32 independent MFMAs per round (each accumulator once per round)
// MODE 1: 32 accumulators, each gets two MFMAs back to back (the hi, lo order of a k-step written per accumulator)
// MODE 2: 8 accumulators only (dependent distance 8)
template <int MODE, int NW>
__global__ __launch_bounds__(NW * 64) void k(int iters, float *out)
{
    const int lane = threadIdx.x & 63;
    bf16x8_t a[4], b[2];
    for (int i = 0; i < 4; i++) for (int e = 0; e < 8; e++) a[i][e] = (__bf16)(0.001f * (lane + i + e));
    for (int i = 0; i < 2; i++) for (int e = 0; e < 8; e++) b[i][e] = (__bf16)(0.002f * (lane - i - e));
    f32x4_t acc[32];
    for (int i = 0; i < 32; i++) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; it++) {
        if (MODE == 0) {
#pragma unroll
            for (int h = 0; h < 2; h++)
#pragma unroll
                for (int i = 0; i < 32; i++) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[h], acc[i], 0, 0, 0);
        } else if (MODE == 1) {
#pragma unroll
            for (int i = 0; i < 32; i++) {
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[0], acc[i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[1], acc[i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 8; h++)
#pragma unroll
                for (int i = 0; i < 8; i++) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[h & 1], acc[i], 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int i = 0; i < 32; i++) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 12345.678f) out[blockIdx.x] = s;
}

template <int MODE, int NW> int run(float *out, hipEvent_t e0, hipEvent_t e1, int grid)
{
    const int iters = 4000;
    float best = 1e9, last = 0;
    for (int rep = 0; rep < 4; rep++) {
        CHK(hipEventRecord(e0));
        hipLaunchKernelGGL((k<MODE, NW>), dim3(grid), dim3(NW * 64), 0, 0, iters, out);
        CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
        float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
        last = ms;
    }
    const double flop = (double)grid * NW * iters * 64 * 16384.0;
    printf("mode %d, %2d waves per workgroup, %4d workgroups: best %8.1f us last %8.1f us  %7.1f TFLOP/s (last %7.1f)\n", MODE, NW, grid, 1e3 * best, 1e3 * last,
           flop / (best * 1e-3) / 1e12, flop / (last * 1e-3) / 1e12);
    fflush(stdout);
    return 0;
}
int main()
{
    float *out; CHK(hipMalloc(&out, 1 << 16)); CHK(hipMemset(out, 0, 1 << 16));
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
    if (run<0, 8>(out, e0, e1, 256)) return 1;
    if (run<0, 4>(out, e0, e1, 256)) return 1;
    if (run<0, 8>(out, e0, e1, 2048)) return 1;     // a longer launch: 8 rounds
    if (run<1, 8>(out, e0, e1, 256)) return 1;
    if (run<2, 8>(out, e0, e1, 256)) return 1;
    if (run<0, 12>(out, e0, e1, 256)) return 1;
    CHK(hipDeviceSynchronize());
    printf("done\n");
    return 0;
}
