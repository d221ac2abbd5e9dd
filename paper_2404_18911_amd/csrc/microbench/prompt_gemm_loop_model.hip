// Stand-alone measurement, not part of the library: a model of the main loop of the 128-row prompt projections
// (gemm_prefill2_body in ../kernels.hip.h) on cache-friendly data, to tell what the loop itself can do from what
// a workgroup does around it.  8 multiplying waves (MFMAs on operands read from LDS; two register sets for
// TW 1 / 2, the plain read-then-multiply order for TW 4) and 4 moving waves (global_load_lds into a ring of NB
// stages, exact vmcnt waits), one barrier per k-step of 32.  Every workgroup of an XCD reads the same weight
// tiles and one of 8 activation regions, 8 passes over 128 k-steps.
// Switches: MOVE (the movers load, or only meet), MULT (0 only meet, 1 read operands, 2 read + multiply with two
// register sets, 3 read + multiply in the TW 4 order).
// Build and run:  hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -o loop_model prompt_gemm_loop_model.hip && ./loop_model
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("ERR %s at %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr int KS = 128;

template <int TW, int NB, int MOVE, int MULT>
__device__ __forceinline__ void body(const u32x4_t *W, const u32x4_t *act, int reps, float *out)
{
    constexpr int NTW = 8 * TW, WA = MULT == 3 ? TW : 2 * TW, WP = MULT == 3 ? 8 : 4, TL = NTW + 16, LPW = TL / 4;
    __shared__ u32x4_t As[NB][NTW][64];
    __shared__ u32x4_t Bs[NB][8][2][64];
    const int t = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    const int xcd = blockIdx.x & 7, rg = (blockIdx.x >> 3) & 7;
    auto meet = [&]() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); __builtin_amdgcn_s_barrier(); asm volatile("" ::: "memory"); };
    const int steps = reps * KS;
    int buf = 0;
    if (wave >= 8) {
        const u32x4_t *src0[LPW];
#pragma unroll
        for (int i = 0; i < LPW; i++) {
            const int j = (wave - 8) + 4 * i;
            if (i < NTW / 4) src0[i] = W + ((size_t)xcd * NTW + j) * KS * 64 + lane;        // the XCD's weight tiles: shared by its workgroups
            else src0[i] = act + ((size_t)rg * 16 + (j - NTW)) * KS * 64 + lane;            // the row group's activation tiles
        }
        auto issue = [&](int ks, int bf) {
            const int kk = ks % KS;
#pragma unroll
            for (int i = 0; i < LPW; i++) {
                const int j = (wave - 8) + 4 * i;
                if (i < NTW / 4) __builtin_amdgcn_global_load_lds(src0[i] + kk * 64, &As[bf][j][0], 16, 0, 0);
                else __builtin_amdgcn_global_load_lds(src0[i] + kk * 64, &Bs[bf][(j - NTW) >> 1][(j - NTW) & 1][0], 16, 0, 0);
            }
        };
        if (MOVE) {
#pragma unroll
            for (int s0 = 0; s0 < NB - 1; s0++) issue(s0, s0);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NB - 2) * LPW) : "memory");
        }
        __syncthreads();
        for (int ks = 0; ks < steps; ks++) {
            if (MOVE) {
                issue(ks + NB - 1, buf >= 1 ? buf - 1 : NB - 1);
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NB - 2) * LPW) : "memory");
            }
            meet();
            buf = buf == NB - 1 ? 0 : buf + 1;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    const int a0 = MULT == 3 ? wave * TW : (wave & 3) * WA, g0 = MULT == 3 ? 0 : (wave >> 2) * WP;
    struct Frag { bf16x8_t av[WA], bh[WP], bl[WP]; };
    f32x4_t acc[WA][WP];
    for (int i = 0; i < WA; i++) for (int j = 0; j < WP; j++) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    auto fetch = [&](Frag &f, int bf) {
#pragma unroll
        for (int i = 0; i < WA; i++) f.av[i] = __builtin_bit_cast(bf16x8_t, As[bf][a0 + i][lane]);
#pragma unroll
        for (int i = 0; i < WP; i++) f.bh[i] = __builtin_bit_cast(bf16x8_t, Bs[bf][g0 + i][0][lane]);
#pragma unroll
        for (int i = 0; i < WP; i++) f.bl[i] = __builtin_bit_cast(bf16x8_t, Bs[bf][g0 + i][1][lane]);
    };
    auto step = [&](const Frag &cur, Frag &nxt) {
        if (MULT == 2) {
#pragma unroll
            for (int j = 0; j < WP; j++)
#pragma unroll
                for (int i = 0; i < WA; i++) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.av[i], cur.bh[j], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        meet();
        buf = buf == NB - 1 ? 0 : buf + 1;
        __builtin_amdgcn_sched_barrier(0);
        if (MULT >= 1) fetch(nxt, buf);
        __builtin_amdgcn_sched_barrier(0);
        if (MULT == 2) {
#pragma unroll
            for (int j = 0; j < WP; j++)
#pragma unroll
                for (int i = 0; i < WA; i++) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.av[i], cur.bl[j], acc[i][j], 0, 0, 0);
        } else if (MULT == 1) {
#pragma unroll
            for (int i = 0; i < WA; i++) asm volatile("" ::"v"(nxt.av[i]));
#pragma unroll
            for (int i = 0; i < WP; i++) asm volatile("" ::"v"(nxt.bh[i]), "v"(nxt.bl[i]));
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    __syncthreads();
    if (MULT == 3) {
        for (int ks = 0; ks < steps; ks++) {
            bf16x8_t av[WA];
#pragma unroll
            for (int i = 0; i < WA; i++) av[i] = __builtin_bit_cast(bf16x8_t, As[buf][a0 + i][lane]);
#pragma unroll
            for (int j = 0; j < WP; j++) {
                const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, Bs[buf][g0 + j][0][lane]);
                const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, Bs[buf][g0 + j][1][lane]);
#pragma unroll
                for (int i = 0; i < WA; i++) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[i], bh, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[i], bl, acc[i][j], 0, 0, 0);
                }
            }
            meet();
            buf = buf == NB - 1 ? 0 : buf + 1;
        }
    } else {
    Frag fa, fb;
    fetch(fa, 0);
    for (int ks = 0; ks < steps; ks += 2) { step(fa, fb); step(fb, fa); }
    }
    float s = 0.f;
    for (int i = 0; i < WA; i++) for (int j = 0; j < WP; j++) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    if (s == 12345.678f) out[blockIdx.x] = s;
}

#define KDEF(TW, NB, MV, ML) __global__ __launch_bounds__(768) void k_##TW##_##NB##_##MV##_##ML(const u32x4_t *W, const u32x4_t *act, int reps, float *out) { body<TW, NB, MV, ML>(W, act, reps, out); }
KDEF(2, 4, 0, 2) KDEF(2, 4, 1, 0) KDEF(2, 4, 1, 1) KDEF(2, 4, 1, 2)
KDEF(1, 6, 0, 2) KDEF(1, 6, 1, 0) KDEF(1, 6, 1, 1) KDEF(1, 6, 1, 2)
KDEF(4, 3, 0, 3) KDEF(4, 3, 1, 0) KDEF(4, 3, 1, 3)
typedef void (*kern_t)(const u32x4_t *, const u32x4_t *, int, float *);
int run(kern_t kern, int TW, int NB, int MOVE, int MULT, const u32x4_t *W, const u32x4_t *act, float *out, hipEvent_t e0, hipEvent_t e1)
{
    const int reps = 8, grid = 256;
    float best = 1e9;
    for (int rep = 0; rep < 3; rep++) {
        CHK(hipEventRecord(e0));
        hipLaunchKernelGGL(kern, dim3(grid), dim3(768), 0, 0, W, act, reps, out);
        CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
        float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    const double steps = (double)reps * KS;
    printf("TW %d NB %d movers %d multipliers %d: %8.1f us  %6.0f ns per step  (matrix work alone %4.0f ns at 2.4 GHz; %5.1f KB moved per step)\n", TW, NB, MOVE, MULT,
           1e3 * best, 1e6 * best / steps, 2.0 * 2 * TW * 4 * 2 * 16 / 2.4, (8 * TW + 16) * 1.0);
    fflush(stdout);
    return 0;
}
int main()
{
    u32x4_t *W, *act; float *out;
    const size_t wbytes = (size_t)8 * 32 * KS * 1024, abytes = (size_t)8 * 16 * KS * 1024;
    CHK(hipMalloc(&W, wbytes)); CHK(hipMalloc(&act, abytes)); CHK(hipMalloc(&out, 1 << 16));
    CHK(hipMemset(W, 0x3c, wbytes)); CHK(hipMemset(act, 0x3c, abytes)); CHK(hipMemset(out, 0, 1 << 16));
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
#define ALL(TW, NB) \
    if (run(k_##TW##_##NB##_0_2, TW, NB, 0, 2, W, act, out, e0, e1)) return 1; \
    if (run(k_##TW##_##NB##_1_0, TW, NB, 1, 0, W, act, out, e0, e1)) return 1; \
    if (run(k_##TW##_##NB##_1_1, TW, NB, 1, 1, W, act, out, e0, e1)) return 1; \
    if (run(k_##TW##_##NB##_1_2, TW, NB, 1, 2, W, act, out, e0, e1)) return 1;
    ALL(2, 4)
    if (run(k_4_3_0_3, 4, 3, 0, 3, W, act, out, e0, e1)) return 1;
    if (run(k_4_3_1_0, 4, 3, 1, 0, W, act, out, e0, e1)) return 1;
    if (run(k_4_3_1_3, 4, 3, 1, 3, W, act, out, e0, e1)) return 1;
    CHK(hipDeviceSynchronize());
    printf("done\n");
    return 0;
}
