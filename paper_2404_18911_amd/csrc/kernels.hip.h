// Device code of libkangaroo: hand-written HIP kernels for gfx950 (CDNA4, 64-wide wavefronts).
//
// Every decode forward of Kangaroo (draft step of M^s = A o M^b[:l], verification by M^b[l:],
// Sections 3.1-3.2 and Figure 2) has at most 8 rows, so each projection is a weight-streaming
// product bounded by HBM bandwidth (Section 1).  The design here:
//   * weights are re-tiled once at load time into 1 KB tiles of 16 rows x 32 k in exactly the
//     register layout of the A operand of v_mfma_f32_16x16x32_bf16, so a wavefront streams
//     contiguous memory with 16-byte loads straight into MFMA operands (no LDS, no conversion);
//   * activations stay fp32; a row is split into bf16 hi + bf16 lo parts that occupy columns
//     m and m+8 of the 16-column B operand, so one MFMA gives fp32-grade products for 8 rows;
//   * the result for a row never depends on how many other rows are in the batch, which keeps
//     verification bit-identical to one-token decoding (needed for token-exact losslessness);
//   * RMSNorm is folded in: the producer's epilogue stores x*g (hi/lo) and per-tile sums of
//     squares, the consumer's epilogue multiplies by rsqrt(mean square + eps).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

#define KG_ROWS 8

enum { EPI_PLAIN = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_HEAD = 3, EPI_SILU = 4 };

// What a projection kernel does with a finished 16-row tile y[16][8].
struct Epi {
    int kind;
    int M;              // live rows (<= 8)
    int N;              // output features of this projection
    // RMSNorm scale of the projection's input rows: rsqrt(sum(ssq_in[t][m]) * inv_d + eps); null = 1
    const float *ssq_in;
    int nt_in;
    float inv_d, eps;
    const float *scale_in;  // prompt passes in 128-row workgroups: the scales themselves, one per row (pf_rms_scale_kernel)
    // EPI_PLAIN: out[(m + row_shift)][n] = y * scale, rows with m + row_shift < 0 are dropped
    float *out;
    int row_shift;
    // EPI_HEAD: as EPI_PLAIN, plus per-tile statistics of z * inv_temp for the rows kept:
    // hstat[(row * N / 16 + tile) * 4 + {0,1,2}] = max, sum exp(. - max), arg-max index (as float bits):
    // the statistics of one row lie together, for the block that reduces them
    float *hstat;
    float inv_temp;
    // EPI_RESID: x = res[m][n] + y; xout[m][n] = x; act_out <- x * gain[n]; ssq_out[tile][m] = sum x^2
    const float *res;
    float *xout;
    // EPI_SILU: act_out <- silu(y * scale) at K index n (the first map of the two-linear-map adapter)
    // EPI_RESID / EPI_SWIGLU: activation for the next projection (K index = n, or tile*8+i for SwiGLU)
    void *act_out;
    int act_pair;       // prompt passes: layout of act_out, see pf_act_ptr (0 = the 8-row layout above)
    int act_K;
    const float *gain;
    float *ssq_out;
};

__device__ __forceinline__ uint16_t f2bf(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// A value the compiler must materialise in a register: what is computed from it cannot be fused
// with what computed it (a * b + c stays a rounded product followed by a sum), so that the same
// source expression rounds alike in every kernel it is written in.
__device__ __forceinline__ float rounded(float v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// device-scope relaxed accesses for data exchanged between workgroups inside one kernel
__device__ __forceinline__ void st_dev(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Store activation value v of row m, feature k, for a consumer projection with K features.
// BF: bf16 hi/lo parts in 1 KB tiles per 32 features, [k/32][row m][part hi|lo][k%32/8][k%8]: the
// 128 bytes of one batch row and k-step are contiguous, so a wave that needs M rows touches M cache
// lines per tile.  MFMA lane (g = lane/16, column j) reads slot ((j%8)*2 + j/8)*4 + g, see b_slot().
// else: plain float [m][K].
template <bool BF>
__device__ __forceinline__ void store_act(void *buf, int K, int m, int k, float v)
{
    if (BF) {
        // the low part is taken from the rounded fp32 value v (fused with a product that made v it
        // would use the unrounded product, and then depend on the caller's expression)
        v = rounded(v);
        uint16_t hi = f2bf(v);
        uint16_t lo = f2bf(v - bf2f(hi));
        uint16_t *p = (uint16_t *)buf;
        size_t base = (size_t)(k >> 5) * 512 + (size_t)(m * 8 + ((k >> 3) & 3)) * 8 + (k & 7);
        p[base] = hi;
        p[base + 32] = lo;
    } else {
        ((float *)buf)[(size_t)m * K + k] = v;
    }
}
// 16-byte slot of MFMA lane `lane` inside a B-operand tile (column j < 8: hi part of row j; j >= 8: lo part of row j-8)
__device__ __forceinline__ int b_slot(int lane) { return (((lane & 7) * 2 + ((lane >> 3) & 1)) << 2) + (lane >> 4); }

// scale[m] = rsqrt(mean square of the input row + eps), from per-tile partial sums, fixed order.
// Wave w of an 8-wave block serves batch row w.  The partials (at most 8 per lane: d <= 8192) are
// fetched by scale_fetch at kernel start so that their latency hides behind the weight stream;
// scale_finish reduces them.  Result valid after the next __syncthreads().
struct ScaleRegs { float v[8]; };
__device__ __forceinline__ void scale_fetch(const float *ssq_in, int M, int nt_in, ScaleRegs &r)
{
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        int i = lane + 64 * j;
        r.v[j] = (ssq_in && wave < M && i < nt_in) ? ssq_in[(size_t)i * KG_ROWS + wave] : 0.f;
    }
}
__device__ __forceinline__ void scale_fetch(const Epi &e, ScaleRegs &r) { scale_fetch(e.ssq_in, e.M, e.nt_in, r); }
__device__ __forceinline__ void scale_finish(const Epi &e, const ScaleRegs &r, float *sc)
{
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave < e.M) {
        float s = 1.f;
        if (e.ssq_in) {
            s = 0.f;
#pragma unroll
            for (int j = 0; j < 8; j++) s += r.v[j];
            for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
            s = rsqrtf(fmaf(s, e.inv_d, e.eps));
        }
        if (lane == 0) sc[wave] = s;
    }
}
// for blocks with fewer than 8 waves
__device__ __forceinline__ void compute_scale(const Epi &e, float *sc)
{
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int m = wave; m < e.M; m += (int)(blockDim.x >> 6)) {
        float s = 1.f;
        if (e.ssq_in) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                int i = lane + 64 * j;
                v[j] = i < e.nt_in ? e.ssq_in[(size_t)i * KG_ROWS + m] : 0.f;
            }
            s = 0.f;
#pragma unroll
            for (int j = 0; j < 8; j++) s += v[j];
            for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
            s = rsqrtf(fmaf(s, e.inv_d, e.eps));
        }
        if (lane == 0) sc[m] = s;
    }
}

// Epilogue on a finished tile: yt[16][8] in LDS (row in tile, batch row), all 256 threads call it.
// Prompt passes: where the producer of a projection's input puts row m of 8-row block b, feature k.
// Returns the address of the hi part; the lo part lies lo_off elements further.
// pair = 0: the block's own tiles [k/32][row m][hi|lo][k%32/8][k%8], what the 8-row kernels read.
// pair = 1: tiles of two blocks, [k/32][hi|lo][lane (8 (b % 2) + m) + 16 (k%32/8)][k%8]: the B operand of a
// 16-row MFMA as one contiguous KB, which a mover wave fetches with one coalesced access per four lanes
// (gathered from the 8-row layout the same tile costs one access per lane: neighbouring lanes then
// read 128 bytes apart).
__device__ __forceinline__ uint16_t *pf_act_ptr(void *base, size_t blk_bytes, int b, int m, int k, int pair, int &lo_off)
{
    uint16_t *p = (uint16_t *)base;
    if (pair) {
        lo_off = 512;
        return p + (size_t)(b >> 1) * blk_bytes + (size_t)(k >> 5) * 1024 + (size_t)(((b & 1) * 8 + m) + 16 * ((k >> 3) & 3)) * 8 + (k & 7);
    }
    lo_off = 32;
    return p + (size_t)b * (blk_bytes >> 1) + (size_t)(k >> 5) * 512 + (size_t)(m * 8 + ((k >> 3) & 3)) * 8 + (k & 7);
}
// one value, split as store_act splits it
__device__ __forceinline__ void store_act_pf(void *base, size_t blk_bytes, int b, int m, int k, float v, int pair)
{
    int lo_off;
    uint16_t *p = pf_act_ptr(base, blk_bytes, b, m, k, pair, lo_off);
    v = rounded(v);
    const uint16_t hi = f2bf(v);
    p[0] = hi;
    p[lo_off] = f2bf(v - bf2f(hi));
}

template <bool BF>
__device__ __forceinline__ void epilogue(const Epi &e, int rt, float (*yt)[KG_ROWS], const float *sc,
                                         float (*sq)[KG_ROWS], float resv = 0.f, float gainv = 1.f,
                                         bool prefetched = false)
{
    int t = threadIdx.x;
    if (e.kind == EPI_PLAIN || e.kind == EPI_HEAD) {
        if (t < 128) {
            int row = t >> 3, m = t & 7;
            int mo = m + e.row_shift;
            float z = yt[row][m] * sc[m];
            if (m < e.M && mo >= 0) e.out[(size_t)mo * e.N + rt * 16 + row] = z;
            sq[row][m] = z * e.inv_temp;
        }
        if (e.kind == EPI_HEAD) {
            __syncthreads();
            int mo = t + e.row_shift;
            if (t < e.M && mo >= 0) {
                float best = sq[0][t];
                int bi = 0;
                for (int r = 1; r < 16; r++)
                    if (sq[r][t] > best) { best = sq[r][t]; bi = r; }
                float sum = 0.f;
                for (int r = 0; r < 16; r++) sum += __expf(sq[r][t] - best);
                float *hs = e.hstat + ((size_t)mo * (e.N >> 4) + rt) * 4;
                hs[0] = best;
                hs[1] = sum;
                hs[2] = __int_as_float(rt * 16 + bi);
            }
        }
    } else if (e.kind == EPI_RESID) {
        if (t < 128) {
            int row = t >> 3, m = t & 7;
            float v = 0.f;
            if (m < e.M) {
                int n = rt * 16 + row;
                if (!prefetched) {
                    resv = e.res[(size_t)m * e.N + n];
                    gainv = e.gain ? e.gain[n] : 1.f;
                }
                v = resv + yt[row][m];
                e.xout[(size_t)m * e.N + n] = v;
                if (e.act_out) store_act<BF>(e.act_out, e.act_K, m, n, e.gain ? v * gainv : v);
            }
            sq[row][m] = v * v;
        }
        if (e.ssq_out) {
            __syncthreads();
            if (t < KG_ROWS) {
                float s = 0.f;
                for (int r = 0; r < 16; r++) s += sq[r][t];
                e.ssq_out[(size_t)rt * KG_ROWS + t] = s;
            }
        }
    } else if (e.kind == EPI_SILU) {
        if (t < 128) {
            int row = t >> 3, m = t & 7;
            if (m < e.M) {
                float g = yt[row][m] * sc[m];
                store_act<BF>(e.act_out, e.act_K, m, rt * 16 + row, g / (1.f + __expf(-g)));
            }
        }
    } else { // EPI_SWIGLU: tile rows (2i, 2i+1) = (gate, up) of feed-forward feature rt*8 + i
        if (t < 64) {
            int i = t >> 3, m = t & 7;
            if (m < e.M) {
                float g = yt[2 * i][m] * sc[m], u = yt[2 * i + 1][m] * sc[m];
                float a = g / (1.f + __expf(-g)) * u;
                store_act<BF>(e.act_out, e.act_K, m, rt * 8 + i, a);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Order of a row tile's KS weight tiles in memory.  The eight waves of a projection block split
// the k-steps into contiguous ranges (wave w starts at ks0(w) = w KS / 8, rounded down) and walk
// them in step; the tiles are stored in the order the block asks for them, the i-th tile of every
// wave next to each other, so that at any moment the block reads one contiguous stretch of memory
// instead of eight stretches KS / 8 KB apart (measured: 18.5 against 19.1 us per projection launch
// at the 7B shape).  Ranges are q = KS / 8 or q + 1 tiles long; the first tile of each of the
// E = KS - 8 q long ranges comes first (in wave order), then the other tiles at E + 8 j + w.
// Which k-steps a wave sums, and in which order, does not depend on where the tiles are stored.
__host__ __device__ __forceinline__ int tile_pos_in_range(int w, int ks, int KS)
{
    const int q = KS >> 3, E = KS - 8 * q;
    const int ks0 = (w * KS) >> 3, len = (((w + 1) * KS) >> 3) - ks0, i = ks - ks0;
    if (len > q) return i == 0 ? ks0 - w * q : E + (i - 1) * 8 + w;
    return E + i * 8 + w;
}
__host__ __device__ __forceinline__ int tile_pos(int ks, int KS) { return tile_pos_in_range((8 * ks + 7) / KS, ks, KS); }

// ---------------------------------------------------------------------------------------------
// Projection, bf16 weights: one block (8 waves) per 16-row tile; the waves split K; each wave
// streams its 1 KB weight tiles with 16-byte non-temporal loads and issues one MFMA per tile.
// W: tiles [rt][tile_pos(ks)][64 lanes][8 bf16]; act: B-operand tiles [ks][64 lanes][8 bf16].

template <int U>
__device__ __forceinline__ void gemv_steps(const u32x4_t *&wp, const u32x4_t *&bp, bool bact, f32x4_t &acc)
{
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    u32x4_t a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; u++) a[u] = __builtin_nontemporal_load(wp + u * 512);
#pragma unroll
    for (int u = 0; u < U; u++) b[u] = bact ? bp[u * 64] : zero;
#pragma unroll
    for (int u = 0; u < U; u++)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[u]),
                                                      __builtin_bit_cast(bf16x8_t, b[u]), acc, 0, 0, 0);
    wp += U * 512;
    bp += U * 64;
}

#define GEMV_WAVES 8

// Everything a wave needs before its first weight load is a leading scalar argument (a copy of the
// fields of e named alike): those arrive preloaded in SGPRs, a field of the by-value struct costs a
// scalar load from the argument block at the start of every launch.
// 14 dwords fit: W, KS, M, act, ssq_in, nt_in, N, res (null unless the epilogue adds a residual), gain.
__global__ __launch_bounds__(64 * GEMV_WAVES, 2) void gemv_bf16_kernel(const u32x4_t *__restrict__ W, int KS, int M,
                                                                   const u32x4_t *__restrict__ act,
                                                                   const float *ssq_in, int nt_in, int N,
                                                                   const float *res, const float *gain, Epi e)
{
    __shared__ float part[GEMV_WAVES][16][KG_ROWS];
    __shared__ float yt[16][KG_ROWS];
    __shared__ float sq[16][KG_ROWS];
    __shared__ float sc[KG_ROWS];
    const int rt = blockIdx.x;
    // The wave index as a scalar, so that everything derived from it (the k range, whether it is a
    // long one) is tested with scalar branches.  This is needed for correctness, not only speed: an
    // MFMA ignores the EXEC mask, and the compiler drops the skip branch around a short
    // exec-masked region, so an `if` on a per-lane copy of a uniform condition that holds nothing
    // but an MFMA executes it also in the waves where the condition is false, on registers those
    // waves never loaded.
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int ks0 = (wave * KS) / GEMV_WAVES, ks1 = ((wave + 1) * KS) / GEMV_WAVES;
    // the wave's tiles sit 8 tiles apart (see tile_pos); a long range has one more tile up front
    const int q = KS >> 3, n_long = KS - 8 * q;
    const bool long_range = ks1 - ks0 > q;
    const u32x4_t *wbase = W + (size_t)rt * KS * 64 + lane;
    const u32x4_t *wp = wbase + (size_t)(n_long + wave) * 64;
    const u32x4_t *bp = act + (size_t)(ks0 + (long_range ? 1 : 0)) * 64 + b_slot(lane);
    const bool bact = (lane & 7) < M;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    ScaleRegs sr;
    scale_fetch(ssq_in, M, nt_in, sr);
    float resv = 0.f, gainv = 1.f;       // epilogue operands of thread (row, m), fetched early
    if (res && threadIdx.x < 128 && (threadIdx.x & 7) < M) {
        int nn = rt * 16 + (threadIdx.x >> 3);
        resv = res[(size_t)(threadIdx.x & 7) * N + nn];
        if (gain) gainv = gain[nn];
    }
    int n = q;
    {
        // chunks of 4 tiles, double-buffered: the loads of chunk i+1 are in flight while chunk i is
        // multiplied, so a wave never drains its memory pipe between chunks
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        u32x4_t a0[4], b0[4], a1[4], b1[4];
        u32x4_t ax = zero, bx = zero;                      // first tile of a long range (k-step ks0)
        if (long_range) {
            ax = __builtin_nontemporal_load(wbase + (size_t)(ks0 - wave * q) * 64);
            if (bact) bx = act[(size_t)ks0 * 64 + b_slot(lane)];
        }
        int rem = n >> 2;
        n &= 3;
#define LD4(A, B)                                                                  \
    {                                                                              \
        _Pragma("unroll") for (int u = 0; u < 4; u++) A[u] = __builtin_nontemporal_load(wp + u * 512); \
        _Pragma("unroll") for (int u = 0; u < 4; u++) B[u] = bact ? bp[u * 64] : zero;                \
        wp += 2048; bp += 256;                                                     \
    }
#define MMA4(A, B)                                                                 \
    _Pragma("unroll") for (int u = 0; u < 4; u++)                                  \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A[u]), __builtin_bit_cast(bf16x8_t, B[u]), acc, 0, 0, 0);
        if (rem) LD4(a0, b0)
        if (long_range)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ax), __builtin_bit_cast(bf16x8_t, bx), acc, 0, 0, 0);
        while (rem >= 2) {
            LD4(a1, b1)
            MMA4(a0, b0)
            if (rem > 2) LD4(a0, b0)
            MMA4(a1, b1)
            rem -= 2;
        }
        if (rem == 1) { MMA4(a0, b0) }
#undef LD4
#undef MMA4
    }
    if (n >= 4) { gemv_steps<4>(wp, bp, bact, acc); n -= 4; }
    if (n >= 2) { gemv_steps<2>(wp, bp, bact, acc); n -= 2; }
    if (n >= 1) { gemv_steps<1>(wp, bp, bact, acc); }
    scale_finish(e, sr, sc);
    // D layout: lane holds column (lane & 15) and tile rows 4*(lane >> 4) + r.  Columns m and m+8
    // are the hi and lo parts of batch row m: fold them.
#pragma unroll
    for (int r = 0; r < 4; r++) {
        float v = acc[r] + __shfl_xor(acc[r], 8);
        if ((lane & 15) < 8) part[wave][4 * (lane >> 4) + r][lane & 7] = v;
    }
    __syncthreads();
    if (threadIdx.x < 128) {
        int row = threadIdx.x >> 3, m = threadIdx.x & 7;
        float v = part[0][row][m];
#pragma unroll
        for (int w = 1; w < GEMV_WAVES; w++) v += part[w][row][m];
        yt[row][m] = v;
    }
    __syncthreads();
    epilogue<true>(e, rt, yt, sc, sq, resv, gainv, true);
}

// The one-row projection on the vector ALUs instead of the matrix units, over the same weight tiles,
// launch shape, k ranges and chunked, double-buffered loads as gemv_bf16_kernel: the comparison that
// backs the choice of an MFMA per tile also at one row (where 7 of its 8 row columns are idle).  A
// lane holds 8 consecutive k of one weight row: it widens them and multiplies by the row's fp32
// activations, the four lanes of a row are added at the end of the wave's range, the waves through LDS.
// y[n] = sum_k W[n][k] x[k], plain fp32 output; used by kg_op_linear_valu only.
__global__ __launch_bounds__(64 * GEMV_WAVES, 2) void gemv_bf16_valu_kernel(const u32x4_t *__restrict__ W, int KS,
                                                                        const float *__restrict__ x, int K, float *y)
{
    __shared__ float part[GEMV_WAVES][16];
    const int rt = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int ks0 = (wave * KS) / GEMV_WAVES, ks1 = ((wave + 1) * KS) / GEMV_WAVES;
    const int q = KS >> 3, n_long = KS - 8 * q;
    const bool long_range = ks1 - ks0 > q;
    const u32x4_t *wbase = W + (size_t)rt * KS * 64 + lane;
    const u32x4_t *wp = wbase + (size_t)(n_long + wave) * 64;
    const int g8 = (lane >> 4) * 8;
    int ks = ks0 + (long_range ? 1 : 0);
    float acc = 0.f;
    auto mac = [&](const u32x4_t &a, int kstep) {
        const int k0 = kstep * 32 + g8;
        float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0;
        if (k0 + 8 <= K) { x0 = *(const float4 *)(x + k0); x1 = *(const float4 *)(x + k0 + 4); }
        acc = fmaf(__uint_as_float(a[0] << 16), x0.x, acc); acc = fmaf(__uint_as_float(a[0] & 0xFFFF0000u), x0.y, acc);
        acc = fmaf(__uint_as_float(a[1] << 16), x0.z, acc); acc = fmaf(__uint_as_float(a[1] & 0xFFFF0000u), x0.w, acc);
        acc = fmaf(__uint_as_float(a[2] << 16), x1.x, acc); acc = fmaf(__uint_as_float(a[2] & 0xFFFF0000u), x1.y, acc);
        acc = fmaf(__uint_as_float(a[3] << 16), x1.z, acc); acc = fmaf(__uint_as_float(a[3] & 0xFFFF0000u), x1.w, acc);
    };
    if (long_range) {
        const u32x4_t ax = __builtin_nontemporal_load(wbase + (size_t)(ks0 - wave * q) * 64);
        mac(ax, ks0);
    }
    int n = q;
    u32x4_t a0[4], a1[4];
    int rem = n >> 2;
    n &= 3;
#define LDV(A) { _Pragma("unroll") for (int u = 0; u < 4; u++) A[u] = __builtin_nontemporal_load(wp + u * 512); wp += 2048; }
#define MACV(A) { _Pragma("unroll") for (int u = 0; u < 4; u++) mac(A[u], ks + u); ks += 4; }
    if (rem) LDV(a0)
    while (rem >= 2) {
        LDV(a1)
        MACV(a0)
        if (rem > 2) LDV(a0)
        MACV(a1)
        rem -= 2;
    }
    if (rem == 1) MACV(a0)
#undef LDV
#undef MACV
    for (; n > 0; n--) {
        const u32x4_t a = __builtin_nontemporal_load(wp);
        wp += 512;
        mac(a, ks++);
    }
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (lane < 16) part[wave][lane] = acc;
    __syncthreads();
    if (threadIdx.x < 16) {
        float v = part[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < GEMV_WAVES; w++) v += part[w][threadIdx.x];
        y[rt * 16 + threadIdx.x] = v;
    }
}

// Projection, fp32 weights (row-major [N][K]) and fp32 activations [8][K]: 16 threads per row.
// Only the small fp32 correctness configuration uses it.
__global__ __launch_bounds__(256) void gemv_f32_kernel(const float *__restrict__ W, int K,
                                                       const float *__restrict__ act, Epi e)
{
    __shared__ float yt[16][KG_ROWS];
    __shared__ float sq[16][KG_ROWS];
    __shared__ float sc[KG_ROWS];
    const int rt = blockIdx.x;
    const int row = threadIdx.x >> 4, sub = threadIdx.x & 15;
    const float *wr = W + (size_t)(rt * 16 + row) * K;
    float acc[KG_ROWS];
#pragma unroll
    for (int m = 0; m < KG_ROWS; m++) acc[m] = 0.f;
    for (int k = sub; k < K; k += 16) {
        float w = wr[k];
#pragma unroll
        for (int m = 0; m < KG_ROWS; m++)
            if (m < e.M) acc[m] = fmaf(w, act[(size_t)m * K + k], acc[m]);
    }
    compute_scale(e, sc);
#pragma unroll
    for (int m = 0; m < KG_ROWS; m++) {
        float v = acc[m];
        for (int o = 8; o >= 1; o >>= 1) v += __shfl_xor(v, o);
        if (sub == 0) yt[row][m] = v;
    }
    __syncthreads();
    epilogue<false>(e, rt, yt, sc, sq);
}

// ---------------------------------------------------------------------------------------------
// Projection for the prompt (prefill): Y[T][N] = X[T][K] . W^T for T up to a few hundred rows, a
// dense contraction on the MFMA units.  Rows are handled in blocks of 8 (hi/lo columns of one
// MFMA, exactly as in decoding), so every output is computed by the same instruction sequence as
// in gemv_bf16_kernel: per output tile the k-steps are split into the same 8 ranges, each range is
// accumulated in order by MFMA, hi and lo are folded, and the 8 range sums are added in order.
// A cache prefilled by this kernel and the 8-row attention is therefore bit-identical to one written
// token by token (the bfloat16 / float32 cache options; with the half-precision cache long passes use
// gemm_prefill2_body and pf_attn_kernel below, which sum in another order).
//   A workgroup handles a group of CBW row blocks (CBW = 8: 64 rows) and a group of 8 * TW weight tiles.
//   It has 12 waves: waves 8..11 only move data, waves 0..7 only multiply.  The movers bring the
//   weight tiles and the activation tiles of a stage (PF_KC k-steps) straight from memory into LDS
//   (global_load_lds: no registers in between), two stages ahead of the multiplication, into a ring
//   of PF_NB stage buffers, and wait with explicit counts for the stage that is due; the
//   multipliers read operands from LDS only, so they never wait on memory.  Wave w of the
//   multipliers owns TW weight tiles and TW * CBW accumulators: every activation tile read from
//   LDS feeds TW MFMAs.  Activation tiles sit in LDS in MFMA lane order (lane l fetches the piece it
//   will use), so a read touches 64 consecutive 16-byte pieces, free of bank conflicts.  Rows
//   beyond the last one of a block are not masked: an MFMA column only depends on its own column of
//   B, and the results of those columns are never stored.
//   The grid is one-dimensional: workgroup id -> (XCD = id % 8, j = id / 8), row group = j % gx,
//   tile group = (j / gx) * 8 + XCD, so the workgroups that stream the same weight tiles for
//   different row groups run next to each other on one XCD and share its L2.
#define PF_KC 2
#define PF_CBW 8
#define PF_NB 3

struct PfArgs {
    const u32x4_t *W;       // weight tiles [NT][tile_pos(ks)][64]
    int KS, NT;
    const u32x4_t *act;     // activation tiles, block b at act + b * act_blk
    size_t act_blk;         // 16-byte units per 8-row block
    int T;                  // rows in this pass
    int ssq_in_blk, ssq_out_blk;   // floats per 8-row block of the sum-of-squares arrays
    size_t act_out_blk;     // bytes per 8-row block of the output activation
    int gx, gy;             // row groups, tile groups (the grid holds gx * 8 * ceil(gy / 8) workgroups)
};

__device__ __forceinline__ Epi pf_block_epi(const Epi &e, const PfArgs &a, int b)
{
    Epi eb = e;
    eb.M = min(KG_ROWS, a.T - 8 * b);
    if (eb.ssq_in) eb.ssq_in += (size_t)b * a.ssq_in_blk;
    if (eb.out) eb.out += (size_t)8 * b * e.N;
    if (eb.res) eb.res += (size_t)8 * b * e.N;
    if (eb.xout) eb.xout += (size_t)8 * b * e.N;
    if (eb.act_out) eb.act_out = (char *)eb.act_out + (size_t)b * a.act_out_blk;
    if (eb.ssq_out) eb.ssq_out += (size_t)b * a.ssq_out_blk;
    return eb;
}

struct PfStage { int r, k, n; };   // k-range index (0..7, 8 = end), first k-step, k-steps in the stage

// the stage that starts at k-step k of range r (or the first stage of the next non-empty range)
__device__ __forceinline__ PfStage pf_stage_at(int r, int k, int KS)
{
    while (r < 8) {
        int k1 = ((r + 1) * KS) >> 3;
        if (k < k1) return PfStage{r, k, min(PF_KC, k1 - k)};
        r++;
        k = (r * KS) >> 3;
    }
    return PfStage{8, 0, 0};
}

template <int PF_TW, int CBW>
__device__ __forceinline__ void gemm_prefill_body(const PfArgs &a, const Epi &e)
{
    constexpr int NTW = 8 * PF_TW;                         // weight tiles of the workgroup
    __shared__ u32x4_t As[PF_NB][PF_KC][NTW][64];
    __shared__ u32x4_t Bs[PF_NB][PF_KC][CBW][64];
    __shared__ float scs[CBW][KG_ROWS];
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const bool mover = wave >= 8;
    const int nb = (a.T + 7) >> 3;
    const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
    const int gyi = (jj / a.gx) * 8 + xcd;
    if (gyi >= a.gy) return;
    const int b0 = (jj % a.gx) * CBW;
    const int nbw = min(CBW, nb - b0);
    const int rt0 = (gyi * 8 + (wave & 7)) * PF_TW;
    const int KS = a.KS;

    // RMS scales of this block group's rows: wave w serves row block w; all partial sums of its 8
    // rows are fetched at once, then every row is reduced exactly as in decoding (lane sums in index
    // order, then the same butterfly)
    static_assert(CBW <= 8, "one wave per row block");
    if (wave < nbw) {
        const Epi eb = pf_block_epi(e, a, b0 + wave);
        float pv[KG_ROWS][8];
#pragma unroll
        for (int m = 0; m < KG_ROWS; m++)
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const int i = lane + 64 * j;
                pv[m][j] = (eb.ssq_in && m < eb.M && i < eb.nt_in) ? eb.ssq_in[(size_t)i * KG_ROWS + m] : 0.f;
            }
#pragma unroll
        for (int m = 0; m < KG_ROWS; m++) {
            float sv = 1.f;
            if (eb.ssq_in) {
                sv = 0.f;
#pragma unroll
                for (int j = 0; j < 8; j++) sv += pv[m][j];
                for (int o = 32; o >= 1; o >>= 1) sv += __shfl_xor(sv, o);
                sv = rsqrtf(fmaf(sv, eb.inv_d, eb.eps));
            }
            if (lane == 0) scs[wave][m] = sv;
        }
    }

    // A stage is up to PF_KC k-steps of one k-range (a range ends a stage early, so the accumulators
    // are folded between stages only).  Per stage the movers issue a fixed number of tile loads
    // (pieces beyond the stage's end, beyond the last weight tile or the last row block read a valid
    // address again; nobody uses them), so the explicit wait counts below are exact.
    constexpr int TL = PF_KC * (NTW + CBW);             // tile loads of a stage
    constexpr int LPW = TL / 4;                            // ... per mover wave
    static_assert(TL % 4 == 0, "tile loads spread evenly over the 4 mover waves");
    bool valid[PF_TW];
#pragma unroll
    for (int tw = 0; tw < PF_TW; tw++) valid[tw] = rt0 + tw < a.NT;
    const int bsl = b_slot(lane);
    // movers: the address of every tile of the wave at k-step 0 is computed once (tile j = wave - 8 + 4 i is
    // uniform in the wave; the first PF_KC * NTW tiles of a stage are weight tiles [kk][tile], the others
    // activation tiles [kk][row block]); a stage then adds the position of its k-steps
    const u32x4_t *src0[LPW];
    if (mover) {
#pragma unroll
        for (int i = 0; i < LPW; i++) {
            const int j = (wave - 8) + 4 * i;
            if (j < PF_KC * NTW) {
                const int rt = min(gyi * NTW + j % NTW, a.NT - 1);
                src0[i] = a.W + (size_t)rt * KS * 64 + lane;
            } else {
                const int cb = (j - PF_KC * NTW) % CBW;
                src0[i] = a.act + (size_t)(b0 + min(cb, nbw - 1)) * a.act_blk + bsl;
            }
        }
    }
    auto issue = [&](const PfStage &sg, int buf) {         // movers: loads of stage sg into ring slot buf
        const int k0 = sg.r < 8 ? sg.k : 0, n = sg.r < 8 ? sg.n : 0;
        int wpos[PF_KC], apos[PF_KC];
#pragma unroll
        for (int kk = 0; kk < PF_KC; kk++) {
            const int ks = k0 + (kk < n ? kk : 0);
            wpos[kk] = tile_pos_in_range(sg.r < 8 ? sg.r : 0, ks, KS) * 64;
            apos[kk] = ks * 64;
        }
#pragma unroll
        for (int i = 0; i < LPW; i++) {
            const int j = (wave - 8) + 4 * i;              // uniform in the wave
            if (j < PF_KC * NTW) {
                const int kk = j / NTW, tile = j % NTW;
                __builtin_amdgcn_global_load_lds(src0[i] + wpos[kk], &As[buf][kk][tile][0], 16, 0, 0);
            } else {
                const int jb = j - PF_KC * NTW, kk = jb / CBW, cb = jb % CBW;
                __builtin_amdgcn_global_load_lds(src0[i] + apos[kk], &Bs[buf][kk][cb][0], 16, 0, 0);
            }
        }
    };
    auto next_of = [&](const PfStage &sg) { return sg.r < 8 ? pf_stage_at(sg.r, sg.k + sg.n, KS) : sg; };

    // The waves meet at bare barriers: the movers wait explicitly for exactly the loads that are due
    // (a fence would wait for all of them, also those issued two stages ahead), and an LDS-direct
    // load has written its tile once it is counted as complete.  Movers and multipliers run loops
    // of their own with the same number of barriers.
    auto meet = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    PfStage cur = pf_stage_at(0, 0, KS), nx1 = next_of(cur);
    int buf = 0;
    if (mover) {
        PfStage nx2 = next_of(nx1);
        issue(cur, 0);
        issue(nx1, 1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW) : "memory");     // the first stage has landed
        __syncthreads();
        while (cur.r < 8) {
            // slot buf + 2 held the stage multiplied before the last barrier; the stage after the
            // current one must have landed before the next barrier
            issue(nx2, buf >= 1 ? buf - 1 : 2);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW) : "memory");
            meet();
            cur = nx1;
            nx1 = nx2;
            nx2 = next_of(nx2);
            buf = buf == PF_NB - 1 ? 0 : buf + 1;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // no load may still be on its way into LDS at the end
        return;
    }
    f32x4_t acc[PF_TW][CBW], tot[PF_TW][CBW];
#pragma unroll
    for (int tw = 0; tw < PF_TW; tw++)
#pragma unroll
        for (int cb = 0; cb < CBW; cb++) {
            acc[tw][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            tot[tw][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }

    __syncthreads();         // first stage in LDS, RMS scales published
    while (cur.r < 8) {
#pragma unroll
        for (int kk = 0; kk < PF_KC; kk++)
            if (kk < cur.n) {
                bf16x8_t av[PF_TW];
#pragma unroll
                for (int tw = 0; tw < PF_TW; tw++) av[tw] = __builtin_bit_cast(bf16x8_t, As[buf][kk][wave * PF_TW + tw][lane]);
#pragma unroll
                for (int cb = 0; cb < CBW; cb++) {
                    const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, Bs[buf][kk][cb][lane]);
#pragma unroll
                    for (int tw = 0; tw < PF_TW; tw++)
                        acc[tw][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[tw], bv, acc[tw][cb], 0, 0, 0);
                }
            }
        if (nx1.r != cur.r) {      // end of a k-range: fold hi/lo, add the range sum in range order
#pragma unroll
            for (int tw = 0; tw < PF_TW; tw++)
#pragma unroll
                for (int cb = 0; cb < CBW; cb++) {
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        float v = acc[tw][cb][r] + __shfl_xor(acc[tw][cb][r], 8);
                        tot[tw][cb][r] = (cur.r == 0) ? v : tot[tw][cb][r] + v;
                    }
                    acc[tw][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                }
            // empty ranges between cur.r and the next stage's contribute exact zeros
        }
        meet();
        cur = nx1;
        nx1 = next_of(nx1);
        buf = buf == PF_NB - 1 ? 0 : buf + 1;
    }

    // Epilogue straight from the accumulators: after the fold, lane (column m = lane % 16 < 8, group
    // g = lane / 16) holds rows 4g..4g+3 of the 16-row tile for batch row m, i.e. four consecutive
    // output features: vector loads and stores, no staging.  Same arithmetic as the one-token epilogue.
    const int col = lane & 15, g4 = lane >> 4;
#pragma unroll
    for (int tw = 0; tw < PF_TW; tw++) {
        const int rt = rt0 + tw;
        const int n0 = rt * 16 + 4 * g4;
        const bool okl = valid[tw] && col < KG_ROWS;
        if (e.kind == EPI_RESID) {
            float4 rv[CBW];
            const float4 gv = (okl && e.gain) ? *(const float4 *)(e.gain + n0) : make_float4(1.f, 1.f, 1.f, 1.f);
#pragma unroll
            for (int cb = 0; cb < CBW; cb++) {
                const int M = min(KG_ROWS, a.T - 8 * (b0 + cb));
                rv[cb] = (okl && cb < nbw && col < M) ? *(const float4 *)(e.res + ((size_t)8 * (b0 + cb) + col) * e.N + n0)
                                                       : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int cb = 0; cb < CBW; cb++) {
                if (cb >= nbw) break;
                const Epi eb = pf_block_epi(e, a, b0 + cb);
                const bool live = okl && col < eb.M;
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (live) {
                    v[0] = rv[cb].x + tot[tw][cb][0]; v[1] = rv[cb].y + tot[tw][cb][1];
                    v[2] = rv[cb].z + tot[tw][cb][2]; v[3] = rv[cb].w + tot[tw][cb][3];
                    *(float4 *)(eb.xout + (size_t)col * eb.N + n0) = make_float4(v[0], v[1], v[2], v[3]);
                    if (eb.act_out) {
                        const float gq[4] = {gv.x, gv.y, gv.z, gv.w};
                        uint16_t hi[4], lo[4];
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            const float x = rounded(eb.gain ? v[r] * gq[r] : v[r]);
                            hi[r] = f2bf(x);
                            lo[r] = f2bf(x - bf2f(hi[r]));
                        }
                        int lo_off;
                        uint16_t *pa = pf_act_ptr(e.act_out, a.act_out_blk, b0 + cb, col, n0, e.act_pair, lo_off);
                        *(uint2 *)pa = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
                        *(uint2 *)(pa + lo_off) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
                    }
                }
                if (eb.ssq_out) {
                    // sum of squares over the 16 rows of the tile in row order: a chain through the 4 lane groups
                    float sq = 0.f;
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const float up = __shfl(sq, (lane & 15) + 16 * (g > 0 ? g - 1 : 0));
                        if (g4 == g) {
                            float c = g ? up : 0.f;
#pragma unroll
                            for (int r = 0; r < 4; r++) c += rounded(v[r] * v[r]);
                            sq = c;
                        }
                    }
                    if (valid[tw] && g4 == 3 && col < KG_ROWS) eb.ssq_out[(size_t)rt * KG_ROWS + col] = sq;
                }
            }
        } else {
#pragma unroll
            for (int cb = 0; cb < CBW; cb++) {
                if (cb >= nbw) break;
                const Epi eb = pf_block_epi(e, a, b0 + cb);
                if (!(okl && col < eb.M)) continue;
                const float sc = scs[cb][col];
                if (eb.kind == EPI_PLAIN) {
                    *(float4 *)(eb.out + (size_t)col * eb.N + n0) =
                        make_float4(tot[tw][cb][0] * sc, tot[tw][cb][1] * sc, tot[tw][cb][2] * sc, tot[tw][cb][3] * sc);
                } else {                          // EPI_SWIGLU: rows (2i, 2i+1) = (gate, up) of feature rt*8 + i
                    uint16_t hi[2], lo[2];
#pragma unroll
                    for (int i = 0; i < 2; i++) {
                        const float g = tot[tw][cb][2 * i] * sc, u = tot[tw][cb][2 * i + 1] * sc;
                        const float av = rounded(g / (1.f + __expf(-g)) * u);
                        hi[i] = f2bf(av);
                        lo[i] = f2bf(av - bf2f(hi[i]));
                    }
                    const int k0 = rt * 8 + 2 * g4;
                    int lo_off;
                    uint16_t *pa = pf_act_ptr(e.act_out, a.act_out_blk, b0 + cb, col, k0, e.act_pair, lo_off);
                    *(uint32_t *)pa = hi[0] | ((uint32_t)hi[1] << 16);
                    *(uint32_t *)(pa + lo_off) = lo[0] | ((uint32_t)lo[1] << 16);
                }
            }
        }
    }
}

// one or two weight tiles per multiplying wave; row groups of PF_CBW blocks, or of 4 for projections
// with so few weight tiles that groups of 8 would leave compute units without a workgroup
__global__ __launch_bounds__(768) void gemm_prefill_kernel_tw1(PfArgs a, Epi e) { gemm_prefill_body<1, PF_CBW>(a, e); }
__global__ __launch_bounds__(768) void gemm_prefill_kernel_tw2(PfArgs a, Epi e) { gemm_prefill_body<2, PF_CBW>(a, e); }
__global__ __launch_bounds__(768) void gemm_prefill_kernel_tw1_cb4(PfArgs a, Epi e) { gemm_prefill_body<1, 4>(a, e); }

// ---------------------------------------------------------------------------------------------
// RMSNorm scale of every row of a prompt pass: rsqrt(sum of the row's tile sums of squares / d + eps),
// the sums taken in the order of the one-token kernels (a lane adds its tiles lane, lane + 64, .., then
// the lanes are folded).  One workgroup per 8-row block, one wave per row; rows beyond the pass get the
// scale of an all-zero row and are not used.
__global__ __launch_bounds__(512) void pf_rms_scale_kernel(const float *ssq, int ssq_blk, int nt_in, int T, float inv_d,
                                                           float eps, float *scale)
{
    const int b = blockIdx.x, m = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int M = min(KG_ROWS, T - KG_ROWS * b);
    const float *p = ssq + (size_t)b * ssq_blk;
    float pv[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int i = lane + 64 * j;
        pv[j] = (m < M && i < nt_in) ? p[(size_t)i * KG_ROWS + m] : 0.f;
    }
    float sv = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) sv += pv[j];
    for (int o = 32; o >= 1; o >>= 1) sv += __shfl_xor(sv, o);
    if (lane == 0) scale[(size_t)b * KG_ROWS + m] = rsqrtf(fmaf(sv, inv_d, eps));
}

// ---------------------------------------------------------------------------------------------
// Projection for long prompt passes: the same contraction as gemm_prefill_body for passes of 256 rows
// and more (where the launch fills at least 45 % of the compute units), organised for reuse instead of
// for the one-token kernel's summation order (a prompt row then differs from the same row decoded alone
// in the order of its sums only, far inside the logit tolerance).  A workgroup owns 8 * TW weight tiles
// x 128 rows.  The hi and lo halves of the activations are two B operands of 16 distinct rows each (two
// 8-row blocks) that are multiplied into the SAME accumulator, so nothing is folded and no per-range
// totals are kept: a weight tile fetched from the L2 serves 128 rows and an activation tile serves up to
// 512 weight rows.  The activations arrive in the pair layout of pf_act_ptr (a B operand = one KB).
//   12 waves: waves 8..11 move, waves 0..7 multiply.  The movers bring the operand tiles of a k-step
// straight into an LDS ring of NB stage buffers (global_load_lds), NB - 1 stages ahead, and wait with
// exact counts; their loop holds nothing but the loads: every tile's address at step 0 is computed
// once, and the k loop walks a row tile's weight tiles in the order they are stored (contiguous memory;
// the sum over k may take any order here) and takes the k-step each one holds from a table, the inverse
// of tile_pos filled at the start, to pick the matching activation tile.
//   PIPE (TW 1, 2): the multiplying waves are arranged 4 x 2, a wave owns 2 TW weight tiles x 4 pairs of
// row blocks (2 TW + 8 operand reads from LDS per 16 TW multiplications instead of TW + 16), all reads
// of a k-step are issued together, the hi halves are multiplied into every accumulator before the lo
// halves, and the operands of k-step ks + 1 are read under the second half of step ks (two register
// sets).  Without PIPE (TW 4, whose 128 accumulator registers leave no room for a second set) a wave
// owns TW weight tiles x all 8 pairs.
#define PF2_KS_MAX 1024
template <int TW, int NB, bool PIPE, int RB = 16>            // RB = 8-row blocks per workgroup: 16, or 8 for launches with few weight tiles
__device__ __forceinline__ void gemm_prefill2_body(const PfArgs &a, const Epi &e)
{
    constexpr int NTW = 8 * TW;
    static_assert(RB == 16 || (RB == 8 && PIPE), "128 rows, or 64 with the 4 x 2 wave arrangement");
    constexpr int WA = PIPE ? 2 * TW : TW;                  // weight tiles of a multiplying wave
    constexpr int WP = PIPE ? RB / 4 : RB / 2;              // its pairs of row blocks (hi and lo operand each)
    __shared__ u32x4_t As[NB][NTW][64];                     // ring of NB stage buffers, one k-step each
    __shared__ u32x4_t Bs[NB][RB / 2][2][64];
    __shared__ float scs[RB][KG_ROWS];
    __shared__ uint16_t kstep_at[PF2_KS_MAX];               // k-step held by the tile at position p of a row tile
    const int t = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    const bool mover = wave >= 8;
    const int nb = (a.T + 7) >> 3;
    const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
    const int gyi = (jj / a.gx) * 8 + xcd;
    if (gyi >= a.gy) return;
    const int b0 = (jj % a.gx) * RB;
    const int nbw = min(RB, nb - b0);
    const int KS = a.KS;
    const int col = lane & 15, g4 = lane >> 4;
    const int a0 = PIPE ? (wave & 3) * WA : wave * TW;      // first weight tile and first pair of a multiplying wave
    const int g0 = PIPE ? ((wave >> 2) & 1) * WP : 0;

    // RMS scales of the group's rows (computed once per pass by pf_rms_scale_kernel: every workgroup summing
    // the tile sums of its 128 rows again cost a tenth of a short pass); the table of k-steps by position
    if (t < nbw * KG_ROWS) scs[t >> 3][t & 7] = e.scale_in ? e.scale_in[(size_t)b0 * KG_ROWS + t] : 1.f;
    for (int i = t; i < KS; i += 768) kstep_at[tile_pos(i, KS)] = (uint16_t)i;
    __syncthreads();

    constexpr int TL = NTW + RB;                            // tile loads of a stage
    constexpr int LPW = TL / 4;
    static_assert(TL % 4 == 0 && NTW % 4 == 0, "tile loads spread evenly over the 4 mover waves, weight tiles first");
    auto meet = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // the movers run NB - 1 stages ahead: when stage ks is multiplied, stages ks + 1 .. ks + NB - 1 are on
    // their way or have landed; after issuing one more, at most NB - 2 stages may still be in flight
    // for the next stage to be complete
    static_assert((NB - 2) * LPW <= 63, "the wait count must fit the instruction's field");
    int buf = 0;
    if (mover) {
        const u32x4_t *src0[LPW];                           // the wave's tiles at k-step 0 (tile j = wave - 8 + 4 i: uniform in the wave)
#pragma unroll
        for (int i = 0; i < LPW; i++) {
            const int j = (wave - 8) + 4 * i;
            if (i < NTW / 4) {
                const int rt = min(gyi * NTW + j, a.NT - 1);
                src0[i] = a.W + (size_t)rt * KS * 64 + lane;
            } else {
                const int jb = j - NTW, grp = jb >> 1, part = jb & 1;
                const int pr = min((b0 >> 1) + grp, (nb - 1) >> 1);
                src0[i] = a.act + (size_t)pr * 2 * a.act_blk + part * 64 + lane;
            }
        }
        auto issue = [&](int ks, int bf) {                  // operands of step ks (clamped: late stages reload a valid one)
            const int kk = min(ks, KS - 1);
            const int wpos = kk * 64, apos = __builtin_amdgcn_readfirstlane((int)kstep_at[kk]) * 128;
#pragma unroll
            for (int i = 0; i < LPW; i++) {
                const int j = (wave - 8) + 4 * i;
                if (i < NTW / 4) __builtin_amdgcn_global_load_lds(src0[i] + wpos, &As[bf][j][0], 16, 0, 0);
                else __builtin_amdgcn_global_load_lds(src0[i] + apos, &Bs[bf][(j - NTW) >> 1][(j - NTW) & 1][0], 16, 0, 0);
            }
        };
#pragma unroll
        for (int s0 = 0; s0 < NB - 1; s0++) issue(s0, s0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NB - 2) * LPW) : "memory");
        __syncthreads();
        for (int ks = 0; ks < KS; ks++) {
            issue(ks + NB - 1, buf >= 1 ? buf - 1 : NB - 1);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NB - 2) * LPW) : "memory");
            meet();
            buf = buf == NB - 1 ? 0 : buf + 1;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    f32x4_t acc[WA][WP];
#pragma unroll
    for (int ta = 0; ta < WA; ta++)
#pragma unroll
        for (int gb = 0; gb < WP; gb++) acc[ta][gb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (PIPE) {
        struct Frag { bf16x8_t av[WA], bh[WP], bl[WP]; };
        auto fetch = [&](Frag &f, int bf) {
#pragma unroll
            for (int ta = 0; ta < WA; ta++) f.av[ta] = __builtin_bit_cast(bf16x8_t, As[bf][a0 + ta][lane]);
#pragma unroll
            for (int gb = 0; gb < WP; gb++) f.bh[gb] = __builtin_bit_cast(bf16x8_t, Bs[bf][g0 + gb][0][lane]);
#pragma unroll
            for (int gb = 0; gb < WP; gb++) f.bl[gb] = __builtin_bit_cast(bf16x8_t, Bs[bf][g0 + gb][1][lane]);
        };
        // Between the halves of a step: the barrier after which stage ks + 1 has landed (and no wave still
        // reads the stage before), and the reads of that stage.
        auto step = [&](const Frag &cur, Frag &nxt) {
#pragma unroll
            for (int gb = 0; gb < WP; gb++)
#pragma unroll
                for (int ta = 0; ta < WA; ta++)
                    acc[ta][gb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.av[ta], cur.bh[gb], acc[ta][gb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            meet();
            buf = buf == NB - 1 ? 0 : buf + 1;
            __builtin_amdgcn_sched_barrier(0);
            fetch(nxt, buf);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int gb = 0; gb < WP; gb++)
#pragma unroll
                for (int ta = 0; ta < WA; ta++)
                    acc[ta][gb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.av[ta], cur.bl[gb], acc[ta][gb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        };
        __syncthreads();
        Frag fa, fb;
        fetch(fa, 0);
        // (the reads after the last step's barrier fetch a stage the movers filled with a valid, unused k-step)
        for (int ks = 0; ks < KS; ks += 2) {
            step(fa, fb);
            if (ks + 1 < KS) step(fb, fa);
        }
    } else {
        __syncthreads();
        for (int ks = 0; ks < KS; ks++) {
            bf16x8_t av[WA];
#pragma unroll
            for (int ta = 0; ta < WA; ta++) av[ta] = __builtin_bit_cast(bf16x8_t, As[buf][a0 + ta][lane]);
#pragma unroll
            for (int gb = 0; gb < WP; gb++) {
                const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, Bs[buf][g0 + gb][0][lane]);
                const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, Bs[buf][g0 + gb][1][lane]);
#pragma unroll
                for (int ta = 0; ta < WA; ta++) {
                    acc[ta][gb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[ta], bh, acc[ta][gb], 0, 0, 0);
                    acc[ta][gb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[ta], bl, acc[ta][gb], 0, 0, 0);
                }
            }
            meet();
            buf = buf == NB - 1 ? 0 : buf + 1;
        }
    }

    // Epilogue from the accumulators: lane (column c, group g4) holds weight rows 4 g4 .. 4 g4 + 3 of a
    // tile for row c % 8 of block b0 + 2 (g0 + gb) + c / 8.
#pragma unroll
    for (int ta = 0; ta < WA; ta++) {
        const int rt = gyi * NTW + a0 + ta;
        const bool valid = rt < a.NT;
        const int n0 = rt * 16 + 4 * g4;
#pragma unroll
        for (int gb = 0; gb < WP; gb++) {
            const int blk = 2 * (g0 + gb) + (col >> 3), m = col & 7;
            const bool in_group = blk < nbw;
            const Epi eb = pf_block_epi(e, a, b0 + min(blk, nbw - 1));
            const bool live = valid && in_group && m < eb.M;
            const f32x4_t y = acc[ta][gb];
            if (e.kind == EPI_RESID) {
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (live) {
                    const float4 rv = *(const float4 *)(eb.res + (size_t)m * eb.N + n0);
                    v[0] = rv.x + y[0]; v[1] = rv.y + y[1]; v[2] = rv.z + y[2]; v[3] = rv.w + y[3];
                    *(float4 *)(eb.xout + (size_t)m * eb.N + n0) = make_float4(v[0], v[1], v[2], v[3]);
                    if (eb.act_out) {
                        const float4 gv = eb.gain ? *(const float4 *)(eb.gain + n0) : make_float4(1.f, 1.f, 1.f, 1.f);
                        const float gq4[4] = {gv.x, gv.y, gv.z, gv.w};
                        uint16_t hi[4], lo[4];
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            const float xv = rounded(v[r] * gq4[r]);
                            hi[r] = f2bf(xv);
                            lo[r] = f2bf(xv - bf2f(hi[r]));
                        }
                        int lo_off;
                        uint16_t *pa = pf_act_ptr(e.act_out, a.act_out_blk, b0 + blk, m, n0, e.act_pair, lo_off);
                        *(uint2 *)pa = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
                        *(uint2 *)(pa + lo_off) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
                    }
                }
                if (e.ssq_out) {                 // sum of squares of the tile's 16 outputs per row: 4 in the lane, then the 4 lane groups
                    float sq = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                    sq += __shfl_xor(sq, 16);
                    sq += __shfl_xor(sq, 32);
                    if (live && g4 == 0) eb.ssq_out[(size_t)rt * KG_ROWS + m] = sq;
                }
            } else if (live) {
                const float sc = scs[blk][m];
                if (e.kind == EPI_PLAIN) {
                    *(float4 *)(eb.out + (size_t)m * eb.N + n0) = make_float4(y[0] * sc, y[1] * sc, y[2] * sc, y[3] * sc);
                } else {                          // EPI_SWIGLU: rows (2i, 2i+1) = (gate, up) of feature rt*8 + i
                    uint16_t hi[2], lo[2];
#pragma unroll
                    for (int i = 0; i < 2; i++) {
                        const float gt = y[2 * i] * sc, up = y[2 * i + 1] * sc;
                        const float av2 = rounded(gt / (1.f + __expf(-gt)) * up);
                        hi[i] = f2bf(av2);
                        lo[i] = f2bf(av2 - bf2f(hi[i]));
                    }
                    const int k0 = rt * 8 + 2 * g4;
                    int lo_off;
                    uint16_t *pa = pf_act_ptr(e.act_out, a.act_out_blk, b0 + blk, m, k0, e.act_pair, lo_off);
                    *(uint32_t *)pa = hi[0] | ((uint32_t)hi[1] << 16);
                    *(uint32_t *)(pa + lo_off) = lo[0] | ((uint32_t)lo[1] << 16);
                }
            }
        }
    }
}
__global__ __launch_bounds__(768) void gemm_prefill2_kernel_tw1(PfArgs a, Epi e) { gemm_prefill2_body<1, 6, true>(a, e); }
__global__ __launch_bounds__(768) void gemm_prefill2_kernel_tw2(PfArgs a, Epi e) { gemm_prefill2_body<2, 4, true>(a, e); }
__global__ __launch_bounds__(768) void gemm_prefill2_kernel_tw4(PfArgs a, Epi e) { gemm_prefill2_body<4, 3, false>(a, e); }
__global__ __launch_bounds__(768) void gemm_prefill2_kernel_tw1_rb8(PfArgs a, Epi e) { gemm_prefill2_body<1, 8, true, 8>(a, e); }

// ---------------------------------------------------------------------------------------------
// Rows -> activation for the first projection of a stack: x[m] = E[tok[m]] (emb != null) or the
// given fp32 rows; writes xout (optional), act = x * gain (hi/lo), ssq[tile][m].  One block per
// 16 features.
struct Tok8 { int t[KG_ROWS]; int vocab; };   // token ids given by the host; vocab bounds the ids read from device memory too

template <bool BF>
__global__ __launch_bounds__(128) void pack_rows_kernel(const void *emb, Tok8 tok, const int *tok_dev,
                                                        const float *rows, int d, int M, const float *gain,
                                                        float *xout, void *act, float *ssq,
                                                        size_t act_blk_bytes = 0, int ssq_blk = 0, int act_pair = 0)
{
    __shared__ float sq[16][KG_ROWS];
    // blockIdx.y selects a block of 8 rows (prefill passes many blocks in one launch; M is then the
    // total row count and every per-row pointer advances by 8 rows per block)
    const int blk = blockIdx.y;
    void *const act_base = act;
    if (blk) {
        M -= 8 * blk;
        if (tok_dev) tok_dev += 8 * blk;
        if (rows) rows += (size_t)8 * blk * d;
        if (xout) xout += (size_t)8 * blk * d;
        act = (char *)act + (size_t)blk * act_blk_bytes;
        if (ssq) ssq += (size_t)blk * ssq_blk;
    }
    if (M > KG_ROWS) M = KG_ROWS;
    int rt = blockIdx.x, row = threadIdx.x >> 3, m = threadIdx.x & 7;
    int n = rt * 16 + row;
    float v = 0.f;
    if (m < M) {
        if (emb) {
            // token ids from the host or from device memory; an id a kernel produced from non-finite
            // logits may be anything: it is clamped so that the gather stays inside the table (the host
            // reports the bad token)
            const int id = min(max(tok_dev ? tok_dev[m] : tok.t[m], 0), tok.vocab - 1);
            size_t idx = (size_t)id * d + n;
            v = BF ? bf2f(((const uint16_t *)emb)[idx]) : ((const float *)emb)[idx];
        } else {
            v = rows[(size_t)m * d + n];
        }
        if (xout) xout[(size_t)m * d + n] = v;
        if (BF && act_pair) store_act_pf(act_base, act_blk_bytes, blk, m, n, gain ? v * gain[n] : v, 1);
        else store_act<BF>(act, d, m, n, gain ? v * gain[n] : v);
    }
    sq[row][m] = v * v;
    __syncthreads();
    if (threadIdx.x < KG_ROWS && ssq) {
        float s = 0.f;
        for (int r = 0; r < 16; r++) s += sq[r][threadIdx.x];
        ssq[(size_t)rt * KG_ROWS + threadIdx.x] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// Weight re-tiling.  Destination row of source row r: mode 0: row_off + r; mode 1 (gate): 16*(r/8)
// + 2*(r%8); mode 2 (up): the same + 1, so a tile holds 8 (gate, up) pairs.
__device__ __forceinline__ int map_row(int r, int row_off, int mode)
{
    return mode == 0 ? row_off + r : 16 * (r >> 3) + 2 * (r & 7) + (mode - 1);
}

__global__ void pack_w_bf16_kernel(const uint16_t *src, int rows, int K, u32x4_t *dst, int KS, int row_off,
                                   int mode)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)rows * KS * 4;
    if (i >= total) return;
    int g = (int)(i & 3);
    int ks = (int)((i >> 2) % KS);
    int r = (int)((i >> 2) / KS);
    int k0 = ks * 32 + g * 8;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (k0 + 8 <= K) v = *(const u32x4_t *)(src + (size_t)r * K + k0);
    int R = map_row(r, row_off, mode);
    dst[((size_t)(R >> 4) * KS + tile_pos(ks, KS)) * 64 + g * 16 + (R & 15)] = v;
}

__global__ void pack_w_f32_kernel(const float *src, int rows, int K, float *dst, int row_off, int mode)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * K) return;
    int r = (int)(i / K), k = (int)(i % K);
    dst[(size_t)map_row(r, row_off, mode) * K + k] = src[i];
}

__global__ void gain_to_f32_kernel(const void *src, int bf, int n, float *dst)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = bf ? bf2f(((const uint16_t *)src)[i]) : ((const float *)src)[i];
}

// cos/sin table of the rotary embedding, angle = pos * inv_freq[i] evaluated in double.
__global__ void rope_table_kernel(float2 *tab, int max_seq, int half, const double *inv_freq)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= max_seq * half) return;
    double a = (double)(i / half) * inv_freq[i % half];
    tab[i] = make_float2((float)cos(a), (float)sin(a));
}

// ---------------------------------------------------------------------------------------------
// Decode attention over a paged KV cache for up to 8 query rows at positions pos0..pos0+M-1.
// grid = (heads, pages in use, blocks of 8 rows); block = 512.  A block handles one head and one
// page of P positions: it rotates q (and k), appends the new k/v rows that fall in its page,
// computes scores, a page-local softmax and P.V, and stores an unnormalised partial.  The last
// block to finish for a head merges the partials in page order (so results do not depend on
// arrival order, nor on how many rows or trailing pages the launch had).
// The argument block is only read (never indexed dynamically, never modified): it then stays in
// scalar registers instead of being copied to private memory.
struct AttnArgs {
    const float *qkv;   // [M][3d]: q | k | v, already RMS-scaled projections
    int d, H, M, pos0, P, logP;
    const int *page_table;
    int pages[16];      // copy of the first 16 page-table entries (saves a dependent load)
    void *kv;           // pool: [phys page][slot][head][K|V][P][hd]
    int slot, n_slots;
    const float2 *rope; // [max_seq][hd/2]
    float *opart;       // [row block][H][S][8][hd]
    float *mxs, *sms;   // [row block][H][S][8]
    int *cnt;           // [row block][H], zero between launches
    int S;              // pages covered by this launch = ceil((pos0+M)/P)
    void *act_out;      // attention output as activation for the output projection (K = d)
    int append_only;    // 1: only append k/v
    // prefill: blockIdx.z selects a block of 8 rows; M is then the total row count
    size_t act_blk_bytes;   // bytes per 8-row block of act_out
    int preappended;    // 1: this call's k/v rows are already in the cache (appended by an earlier launch)
    int append_all;     // with append_only: write every row of the block to its own page (grid.y = 1)
};

// Element types of the KV cache: float, uint16_t (bfloat16 bit patterns), kvhalf_t (IEEE half bit
// patterns).  Keys and values are O(1) numbers, far inside the half range; half keeps three more
// significant bits than bfloat16 in the same two bytes.
// A half only ever exists as an integer bit pattern in memory, registers and aggregates here, and is
// converted at the point of use (arrays of structs with a _Float16 member that are filled
// conditionally came out of the compiler with every second element undefined).
struct kvhalf_t { uint16_t bits; };
static_assert(sizeof(kvhalf_t) == 2, "two-byte cache element");
__device__ __forceinline__ float half_bits_to_f32(uint32_t low16) { return (float)__builtin_bit_cast(_Float16, (uint16_t)low16); }
__device__ __forceinline__ uint16_t f32_to_half_bits(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }
template <typename T> __device__ __forceinline__ float kv_ld(const T *p);
template <> __device__ __forceinline__ float kv_ld<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float kv_ld<uint16_t>(const uint16_t *p) { return bf2f(*p); }
template <> __device__ __forceinline__ float kv_ld<kvhalf_t>(const kvhalf_t *p) { return half_bits_to_f32(p->bits); }
template <typename T> __device__ __forceinline__ float kv_round(float v);     // value as the cache type holds it
template <> __device__ __forceinline__ float kv_round<float>(float v) { return v; }
template <> __device__ __forceinline__ float kv_round<uint16_t>(float v) { return bf2f(f2bf(v)); }
template <> __device__ __forceinline__ float kv_round<kvhalf_t>(float v) { return half_bits_to_f32(f32_to_half_bits(rounded(v))); }
template <typename T> __device__ __forceinline__ void kv_st(T *p, float v);
template <> __device__ __forceinline__ void kv_st<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void kv_st<uint16_t>(uint16_t *p, float v) { *p = f2bf(v); }
template <> __device__ __forceinline__ void kv_st<kvhalf_t>(kvhalf_t *p, float v) { p->bits = f32_to_half_bits(v); }

template <typename T, int N8> struct KvVec;           // N8 groups of 8 cache elements, loaded as 16-byte pieces
template <int N8> struct KvVec<uint16_t, N8> {
    u32x4_t r[N8];
    __device__ __forceinline__ void load(const uint16_t *p)
    {
#pragma unroll
        for (int i = 0; i < N8; i++) r[i] = *(const u32x4_t *)(p + 8 * i);
    }
    __device__ __forceinline__ float get(int i) const
    {
        uint32_t w = r[i >> 3][(i >> 1) & 3];
        return __uint_as_float((i & 1) ? (w & 0xFFFF0000u) : (w << 16));
    }
};
template <int N8> struct KvVec<kvhalf_t, N8> {
    u32x4_t r[N8];
    __device__ __forceinline__ void load(const kvhalf_t *p)
    {
#pragma unroll
        for (int i = 0; i < N8; i++) r[i] = *(const u32x4_t *)(p + 8 * i);
    }
    __device__ __forceinline__ float get(int i) const
    {
        const uint32_t w = r[i >> 3][(i >> 1) & 3];
        return half_bits_to_f32((i & 1) ? (w >> 16) : (w & 0xFFFFu));
    }
};
template <int N8> struct KvVec<float, N8> {
    float4 r[2 * N8];
    __device__ __forceinline__ void load(const float *p)
    {
#pragma unroll
        for (int i = 0; i < 2 * N8; i++) r[i] = *(const float4 *)(p + 4 * i);
    }
    __device__ __forceinline__ float get(int i) const
    {
        const float4 &v = r[i >> 2];
        return (i & 3) == 0 ? v.x : (i & 3) == 1 ? v.y : (i & 3) == 2 ? v.z : v.w;
    }
};

// E consecutive cache elements owned by one lane in the P.V pass (E = head_dim / 64)
template <typename T, int E> struct KvLane;
template <> struct KvLane<uint16_t, 2> {
    uint32_t r;
    __device__ __forceinline__ void load(const uint16_t *p) { r = *(const uint32_t *)p; }
    __device__ __forceinline__ float get(int e) const { return __uint_as_float(e ? (r & 0xFFFF0000u) : (r << 16)); }
};
template <> struct KvLane<uint16_t, 1> {
    uint16_t r;
    __device__ __forceinline__ void load(const uint16_t *p) { r = *p; }
    __device__ __forceinline__ float get(int) const { return bf2f(r); }
};
template <> struct KvLane<kvhalf_t, 2> {
    uint32_t r;
    __device__ __forceinline__ void load(const kvhalf_t *p) { r = *(const uint32_t *)p; }
    __device__ __forceinline__ float get(int e) const { return half_bits_to_f32(e ? (r >> 16) : (r & 0xFFFFu)); }
};
template <> struct KvLane<kvhalf_t, 1> {
    uint32_t r;
    __device__ __forceinline__ void load(const kvhalf_t *p) { r = p->bits; }
    __device__ __forceinline__ float get(int) const { return half_bits_to_f32(r); }
};
template <> struct KvLane<float, 2> {
    float2 r;
    __device__ __forceinline__ void load(const float *p) { r = *(const float2 *)p; }
    __device__ __forceinline__ float get(int e) const { return e ? r.y : r.x; }
};
template <> struct KvLane<float, 1> {
    float r;
    __device__ __forceinline__ void load(const float *p) { r = *p; }
    __device__ __forceinline__ float get(int) const { return r; }
};

// physical page of logical page s: the first 16 come from the argument block through a chain of
// selects on constant indices
__device__ __forceinline__ int attn_page(const AttnArgs &a, int s)
{
    if (s >= 16) return a.page_table[s];
    int p = a.pages[0];
#pragma unroll
    for (int i = 1; i < 16; i++) p = (s == i) ? a.pages[i] : p;
    return p;
}

// Lane exchanges of the softmax reductions as data-parallel-primitive moves (no trip through the
// LDS crossbar as __shfl_xor takes).  All 64 lanes must be active.  quad_x1 / quad_x2: the value of
// lane ^ 1 / lane ^ 2.  half_mirror / row_mirror: the value of the mirrored lane inside a group of
// 8 / 16 lanes; where the value is already uniform over groups of 4 / 8 lanes that is the value
// lane ^ 4 / lane ^ 8 holds, so a butterfly built from them gives every lane the bits the xor
// butterfly gives.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float quad_x1(float v) { return dpp_move<0xB1>(v); }       // quad_perm [1,0,3,2]
__device__ __forceinline__ float quad_x2(float v) { return dpp_move<0x4E>(v); }       // quad_perm [2,3,0,1]
__device__ __forceinline__ float half_mirror(float v) { return dpp_move<0x141>(v); }
__device__ __forceinline__ float row_mirror(float v) { return dpp_move<0x140>(v); }
__device__ __forceinline__ float lane_value(float v, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
// max / sum over the wave of a value that is uniform over groups of 4 lanes, in the order of the
// xor butterfly over offsets 4, 8, 16, 32 (the last two levels combine the four 16-lane rows as
// (r0 . r1) . (r2 . r3), which is what every lane of that butterfly ends with)
__device__ __forceinline__ float wave_max_q4(float v)
{
    v = fmaxf(v, half_mirror(v));
    v = fmaxf(v, row_mirror(v));
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ float wave_sum_q4(float v)
{
    v += half_mirror(v);
    v += row_mirror(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

// rotation of the pair (x0, x1) by the angle whose (cos, sin) is cs; written with explicit fused
// operations so that every instantiation rounds alike
__device__ __forceinline__ float rot_lo(float x0, float x1, float2 cs) { return fmaf(x0, cs.x, -__fmul_rn(x1, cs.y)); }
__device__ __forceinline__ float rot_hi(float x0, float x1, float2 cs) { return fmaf(x1, cs.x, __fmul_rn(x0, cs.y)); }

// One (head, page) unit, 512 threads, MR >= number of rows (1, 2, 4 or 8: less code and fewer
// registers for the common one- and two-row calls; a row's arithmetic is the same in all of them).
// Scores: 4 lanes per position (a quarter of the head dimension each), all 128 positions of a
// page in one pass.  P.V: a wave walks its 16 positions, every lane owning head_dim/64 output
// elements (no cross-lane reduction).  Softmax statistics are kept per wave, then merged across
// the 8 waves, then across pages; every level rescales by exp(max_part - max_all), in a fixed
// order, so a row's result does not depend on the other rows of the batch or on trailing pages.
template <typename T, int HD, bool BF, int MR>
__global__ __launch_bounds__(512, (sizeof(T) == 2 ? 6 : 1)) void attn_kernel(const AttnArgs a)
{
    constexpr int EL = HD / 4;          // elements of one score lane
    constexpr int EPL = HD / 64;        // output elements of one P.V lane
    constexpr int HH = HD / 2;
    __shared__ __align__(16) float qs[MR][HD];
    __shared__ float kn[MR][HD], vn[MR][HD];     // this call's k, v rows as the cache holds them
    __shared__ float ow[8][MR][HD];
    __shared__ float mw[8][MR], sw[8][MR];
    __shared__ __align__(16) float pw[8][MR][16];   // a wave's probabilities [row][position]
    __shared__ __align__(16) float wtl[MR][8];      // weights of the wave merge [row][wave]
    __shared__ float gml[MR];
    __shared__ int last_flag;
    const int h = blockIdx.x, s = blockIdx.y, zb = blockIdx.z, t = threadIdx.x;
    // the wave index as a scalar: conditions on it (which positions a wave owns) become scalar branches
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    const int P = a.P, d = a.d, logP = a.logP;
    const int pos0 = a.pos0 + 8 * zb;
    const int M = min(MR, a.M - 8 * zb);
    const int S = (pos0 + M + P - 1) >> logP;               // pages this block of rows attends to
    if (!a.append_all && s >= S) return;
    const int hz = zb * a.H + h;                            // index of (row block, head) in the partial buffers
    const float *qkv = a.qkv + (size_t)8 * zb * 3 * d + h * HD;
    const int p_begin = s << logP;
    const int n_valid = min(P, pos0 + M - p_begin);         // positions of this page that hold data
    const int n_old = a.preappended ? n_valid : min(P, max(0, pos0 - p_begin));   // ... cached before this call
    const size_t unit = (size_t)2 * P * HD;                 // K then V of one (page, slot, head)
    T *const Kp = (T *)a.kv + (((size_t)attn_page(a, s) * a.n_slots + a.slot) * a.H + h) * unit;
    T *const Vp = Kp + (size_t)P * HD;
    void *const act_out = (char *)a.act_out + (size_t)zb * a.act_blk_bytes;

    // this call's rows (thread = row rm, rotation pair rj): issued first, they come from the L2
    const bool has_row = t < M * HH;
    const int rm = t / HH, rj = t % HH, rpos = pos0 + rm;
    const bool row_here = has_row && !a.preappended && (a.append_all || (rpos >= p_begin && rpos < p_begin + P));
    float2 cs = make_float2(1.f, 0.f);
    float q0 = 0.f, q1 = 0.f, k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
    if (has_row) {
        const float *q = qkv + (size_t)rm * 3 * d;
        cs = a.rope[(size_t)rpos * HH + rj];
        q0 = q[rj]; q1 = q[rj + HH];
        if (row_here) { k0 = q[d + rj]; k1 = q[d + rj + HH]; v0 = q[2 * d + rj]; v1 = q[2 * d + rj + HH]; }
    }
    // rows cached by earlier calls: score lane (position pl, quarter sub); P.V lane owns EPL elements
    const int pl = t >> 2, sub = t & 3;
    const bool k_old = pl < n_old;
    KvVec<T, EL / 8> kreg;
    KvLane<T, EPL> vreg[16];
    if (!a.append_only) {
        if (k_old) kreg.load(Kp + (size_t)pl * HD + sub * EL);
#pragma unroll
        for (int i = 0; i < 16; i++)
            if (wave * 16 + i < n_old) vreg[i].load(Vp + (size_t)(wave * 16 + i) * HD + EPL * lane);
    }
    if (!has_row && t < MR * HH) { qs[rm][rj] = 0.f; qs[rm][rj + HH] = 0.f; }   // unused rows of the instantiation
    if (has_row) {
        const float qscale = rsqrtf((float)HD);
        qs[rm][rj] = rot_lo(q0, q1, cs) * qscale;
        qs[rm][rj + HH] = rot_hi(q0, q1, cs) * qscale;
        if (row_here) {
            const float ka = kv_round<T>(rot_lo(k0, k1, cs)), kb = kv_round<T>(rot_hi(k0, k1, cs));
            const float va = kv_round<T>(v0), vb = kv_round<T>(v1);
            T *Kq = Kp, *Vq = Vp;
            int pp = rpos - p_begin;
            if (a.append_all) {
                pp = rpos & (P - 1);
                Kq = (T *)a.kv + (((size_t)a.page_table[rpos >> logP] * a.n_slots + a.slot) * a.H + h) * unit;
                Vq = Kq + (size_t)P * HD;
            }
            kv_st<T>(Kq + (size_t)pp * HD + rj, ka);
            kv_st<T>(Kq + (size_t)pp * HD + rj + HH, kb);
            kv_st<T>(Vq + (size_t)pp * HD + rj, va);
            kv_st<T>(Vq + (size_t)pp * HD + rj + HH, vb);
            kn[rm][rj] = ka; kn[rm][rj + HH] = kb;
            vn[rm][rj] = va; vn[rm][rj + HH] = vb;
        }
    }
    if (a.append_only) return;
    __syncthreads();
    // positions written by this call are taken from LDS (the very values the cache now holds)
    const bool k_new = !k_old && pl < n_valid;
    const int mk = p_begin + pl - pos0;

    // scores and wave-local softmax
    // Every row's dot product runs over the lane's EL elements in ascending order; the cached keys
    // are widened once per 4 elements and used for all rows (rows beyond M multiply zeros).
    float pr[MR], dot[MR];
#pragma unroll
    for (int m = 0; m < MR; m++) dot[m] = 0.f;
    if (k_new) {
#pragma unroll
        for (int m = 0; m < MR; m++)
            if (m < M) {
#pragma unroll
                for (int i = 0; i < EL; i++) dot[m] = fmaf(kn[mk][sub * EL + i], qs[m][sub * EL + i], dot[m]);
            }
    } else if (k_old) {
#pragma unroll
        for (int i4 = 0; i4 < EL; i4 += 4) {
            const float kf0 = kreg.get(i4), kf1 = kreg.get(i4 + 1), kf2 = kreg.get(i4 + 2), kf3 = kreg.get(i4 + 3);
#pragma unroll
            for (int m = 0; m < MR; m++) {
                const float4 qv = *(const float4 *)&qs[m][sub * EL + i4];
                dot[m] = fmaf(kf0, qv.x, dot[m]);
                dot[m] = fmaf(kf1, qv.y, dot[m]);
                dot[m] = fmaf(kf2, qv.z, dot[m]);
                dot[m] = fmaf(kf3, qv.w, dot[m]);
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MR; m++) {
        pr[m] = 0.f;
        if (m < M) {
            float v = dot[m];
            v += quad_x1(v);
            v += quad_x2(v);
            const float sc = (pl < n_valid && p_begin + pl <= pos0 + m) ? v : -INFINITY;
            const float mx = wave_max_q4(sc);
            const float p = (mx == -INFINITY) ? 0.f : __expf(sc - mx);
            const float sum = wave_sum_q4(p);
            pr[m] = p;
            if (lane == 0) { mw[wave][m] = mx; sw[wave][m] = sum; }
        }
    }
    // P.V over the wave's 16 positions; the probability of position i sits in lane 4 i
    float acc[MR][EPL];
#pragma unroll
    for (int m = 0; m < MR; m++)
#pragma unroll
        for (int e = 0; e < EPL; e++) acc[m][e] = 0.f;
    // With 4 or 8 rows the wave passes its probabilities through a private LDS row and reads them
    // back four positions at a time as broadcasts (one lane read per (position, row) otherwise:
    // a third of this loop's vector instructions); the products and their order are the same.
    if (MR >= 4) {
        if ((lane & 3) == 0) {
#pragma unroll
            for (int m = 0; m < MR; m++) pw[wave][m][lane >> 2] = pr[m];
        }
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int i4 = 0; i4 < 16; i4 += 4) {
        float4 p4[MR];
        if (MR >= 4) {
#pragma unroll
            for (int m = 0; m < MR; m++) p4[m] = *(const float4 *)&pw[wave][m][i4];
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int i = i4 + j;
            const int pv = wave * 16 + i;
            if (pv < n_valid) {                                  // uniform in the wave
                float vv[EPL];
                if (pv >= n_old) {
#pragma unroll
                    for (int e = 0; e < EPL; e++) vv[e] = vn[p_begin + pv - pos0][EPL * lane + e];
                } else {
#pragma unroll
                    for (int e = 0; e < EPL; e++) vv[e] = vreg[i].get(e);
                }
#pragma unroll
                for (int m = 0; m < MR; m++) {
                    if (MR >= 4) {          // rows beyond M carry probability 0 and are not stored
                        const float p = j == 0 ? p4[m].x : j == 1 ? p4[m].y : j == 2 ? p4[m].z : p4[m].w;
#pragma unroll
                        for (int e = 0; e < EPL; e++) acc[m][e] = fmaf(p, vv[e], acc[m][e]);
                    } else if (m < M) {
                        const float p = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr[m]), 4 * i));
#pragma unroll
                        for (int e = 0; e < EPL; e++) acc[m][e] = fmaf(p, vv[e], acc[m][e]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MR; m++)
        if (m < M) {
#pragma unroll
            for (int e = 0; e < EPL; e++) ow[wave][m][EPL * lane + e] = acc[m][e];
        }
    __syncthreads();
    // merge the 8 waves; a single page is final, otherwise store the page partial
    const bool single = S == 1;
    const size_t pidx = (size_t)hz * a.S + s;
    // weight exp(max_wave - max_all) of every (row, wave), once per block: thread (m, w) = (t / 8, t % 8);
    // a wave without a valid position gets weight 0 (its sums are 0 too)
    if (t < 8 * MR) {
        const float mv = mw[t & 7][t >> 3];
        float gm = mv;
        gm = fmaxf(gm, quad_x1(gm));
        gm = fmaxf(gm, quad_x2(gm));
        gm = fmaxf(gm, half_mirror(gm));
        wtl[t >> 3][t & 7] = (mv == -INFINITY) ? 0.f : __expf(mv - gm);
        if ((t & 7) == 0) gml[t >> 3] = gm;
    }
    __syncthreads();
    for (int i = t; i < M * HD; i += 512) {
        const int m = i / HD, e = i % HD;
        const float gm = gml[m];
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < 8; w++) {
            const float wt = wtl[m][w];
            num = fmaf(wt, ow[w][m][e], num);
            den = fmaf(wt, sw[w][m], den);
        }
        if (single) {
            store_act<BF>(act_out, d, m, h * HD + e, num / den);
        } else {
            st_dev(&a.opart[(pidx * KG_ROWS + m) * HD + e], num);
            if (e == 0) {
                st_dev(&a.mxs[pidx * KG_ROWS + m], gm);
                st_dev(&a.sms[pidx * KG_ROWS + m], den);
            }
        }
    }
    if (single) return;
    // The last block of this head merges the pages in order.  The partials are exchanged with
    // device-scope relaxed atomic stores / loads (write-through, cache-bypassing accesses); every
    // wave waits for its stores to be acknowledged before the block bumps the head's counter.  A
    // device-scope fence would write back and invalidate the whole L2 and costs several
    // microseconds here.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t == 0) {
        const int old = __hip_atomic_fetch_add(&a.cnt[hz], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last_flag = (old == S - 1);
    }
    __syncthreads();
    if (!last_flag) return;
    const size_t hb = (size_t)hz * a.S;
    if (S <= 8) {     // few pages: every load of the merge is issued before any is used
        for (int i = t; i < M * HD; i += 512) {
            const int m = i / HD, e = i % HD;
            float mv[8], ov[8], sv[8];
#pragma unroll
            for (int ss = 0; ss < 8; ss++) {
                const bool in = ss < S;
                mv[ss] = in ? ld_dev(&a.mxs[(hb + ss) * KG_ROWS + m]) : -INFINITY;
                ov[ss] = in ? ld_dev(&a.opart[((hb + ss) * KG_ROWS + m) * HD + e]) : 0.f;
                sv[ss] = in ? ld_dev(&a.sms[(hb + ss) * KG_ROWS + m]) : 0.f;
            }
            float gm = -INFINITY;
#pragma unroll
            for (int ss = 0; ss < 8; ss++) gm = fmaxf(gm, mv[ss]);
            float num = 0.f, den = 0.f;
#pragma unroll
            for (int ss = 0; ss < 8; ss++) {
                if (ss < S) {
                    const float w = (mv[ss] == -INFINITY) ? 0.f : __expf(mv[ss] - gm);
                    num = fmaf(w, ov[ss], num);
                    den = fmaf(w, sv[ss], den);
                }
            }
            store_act<BF>(act_out, d, m, h * HD + e, num / den);
        }
        if (t == 0) __hip_atomic_store(&a.cnt[hz], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    // page weights exp(max_page - max_all), through LDS so that the page loop has independent loads
    float (*wgt)[MR] = (float (*)[MR]) & ow[0][0][0];    // [page][row], S <= 128 <= 8 * HD
    for (int m = wave; m < M; m += 8) {
        float gm = -INFINITY;
        for (int ss = lane; ss < S; ss += 64) gm = fmaxf(gm, ld_dev(&a.mxs[(hb + ss) * KG_ROWS + m]));
        for (int o = 32; o >= 1; o >>= 1) gm = fmaxf(gm, __shfl_xor(gm, o));
        for (int ss = lane; ss < S; ss += 64) {
            const float mxv = ld_dev(&a.mxs[(hb + ss) * KG_ROWS + m]);
            wgt[ss][m] = (mxv == -INFINITY) ? 0.f : __expf(mxv - gm);
        }
    }
    __syncthreads();
    for (int i = t; i < M * HD; i += 512) {
        const int m = i / HD, e = i % HD;
        float num = 0.f, den = 0.f;
        for (int ss = 0; ss < S; ss++) {
            const float w = wgt[ss][m];
            num = fmaf(w, ld_dev(&a.opart[((hb + ss) * KG_ROWS + m) * HD + e]), num);
            den = fmaf(w, ld_dev(&a.sms[(hb + ss) * KG_ROWS + m]), den);
        }
        store_act<BF>(act_out, d, m, h * HD + e, num / den);
    }
    if (t == 0) __hip_atomic_store(&a.cnt[hz], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------------------------
// Attention of the prompt rows (prefill) on the matrix units, for a half-precision KV cache.
// One workgroup per head and block of 64 query rows (4 waves, two workgroups per compute unit) or of
// 128 query rows (8 waves, a compute unit alone, two tiles of K and V in LDS: half the staging per row
// and one barrier per tile; for passes whose blocks of 128 rows fill the device); a wave owns 16 rows.
// The keys and values of all rows of this pass are already in the cache (appended by an earlier
// launch), so the block walks the cache in tiles of 128 positions up to its own last row:
//   S^T = K Q^T   per 16-position tile: A = keys from LDS (as stored: one position's 8 consecutive
//         dimensions per lane), B = the rotated, scaled queries held in registers as half hi + lo
//         parts (two MFMAs per step, fp32-grade scores); the result has a lane's query row in its
//         column and four positions in its registers;
//   row softmax   running maximum and sum per query row (flash-attention recurrence), reductions
//         over a lane's own registers and two lane exchanges;
//   O = P V       A = the probabilities straight from the score registers, rounded to half (the
//         contraction index may be enumerated in any order as long as both operands agree: k-slot
//         j of lane group g is position 32 u + 16 (j / 4) + 4 g + j % 4), B = V^T from LDS, where the
//         values were transposed on the way in and laid out in exactly that order.
// Rows are masked causally; rows beyond the pass are computed and dropped.  The output goes to the
// activation tiles of the output projection (hi + lo bf16 parts per 8-row block), like the decode
// kernel's.  Numerically the rows differ from the decode kernel's in the order of the sums and in
// the half-precision probabilities (relative 2^-12), far inside the logit tolerance.
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

struct PfAttnArgs {
    const float *qkv;        // [T][3d] rows of this pass: q | k | v, RMS-scaled projections, not rotated
    int d, H, T, pos0, logP;
    const int *page_table;
    const kvhalf_t *kv;      // pool: [phys page][slot][head][K|V][P][hd]
    int slot, n_slots;
    const float2 *rope;      // [max_seq][hd/2]
    void *act_out;           // activation tiles of the output projection, one per 8-row block
    size_t act_blk_bytes;
    int act_pair;            // layout of act_out (pf_act_ptr)
};

template <int HD, int NW>     // NW waves: 16 NW query rows per workgroup
__global__ __launch_bounds__(64 * NW, NW == 8 ? 1 : 2) void pf_attn_kernel(const PfAttnArgs a)
{
    constexpr int NT = 64 * NW, ROWS = 16 * NW;
    constexpr int NBUF = NW == 8 ? 2 : 1;       // tiles of K and V^T in LDS (two workgroups of 4 waves share a compute unit instead)
    constexpr int CH = 16 * HD / NT;            // 16-byte chunks of a K tile (and of a V tile) per thread
    constexpr int VSTEP = NT / 128;             // chunk index step of a thread's V chunks
    constexpr int KS = HD / 32;                 // contraction steps of Q.K^T
    constexpr int DT = HD / 16;                 // 16-wide tiles of the head dimension
    constexpr int HH = HD / 2;
    constexpr int KROW = HD + 8;                // halves per key row in LDS (16 bytes of padding: conflict-free 16-byte reads)
    constexpr int VROW = 128 + 8;               // halves per dimension row of V^T in LDS
    __shared__ __align__(16) uint16_t Ks[NBUF][128 * KROW];
    __shared__ __align__(16) uint16_t Vt[NBUF][HD * VROW];
    __shared__ int pages[128];                  // the page table (a context has at most 128 pages)
    const int h = blockIdx.x, t = threadIdx.x;
    const int rb = (int)gridDim.y - 1 - (int)blockIdx.y;        // late row blocks (most tiles) are scheduled first
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    const int q16 = lane & 15, g = lane >> 4;
    const int P = 1 << a.logP, d = a.d;
    const int row = rb * ROWS + wave * 16 + q16;                  // the query row this lane's column stands for
    const int qpos = a.pos0 + row;
    const int last_pos = a.pos0 + min(a.T, rb * ROWS + ROWS) - 1;   // last position any row of the block attends to
    const int n_tiles = (last_pos >> 7) + 1;
    const int wave_last = a.pos0 + min(a.T - 1, rb * ROWS + wave * 16 + 15);
    const size_t unit = (size_t)2 * P * HD;
    if (t <= (last_pos >> a.logP) && t < 128) pages[t] = a.page_table[t];
    __syncthreads();

    // keys as stored: thread -> (position, 8 dimensions); values: thread -> (8 dimensions, position =
    // lane-consecutive).  A tile's loads are issued one tile ahead, into registers, and stay in flight
    // under the multiplications of the tile before.
    u32x4_t kreg[CH], vreg[CH];
    const size_t page_stride = (size_t)a.n_slots * a.H * unit;              // elements per physical page
    const kvhalf_t *kv_head = a.kv + ((size_t)a.slot * a.H + h) * unit;     // this layer's and head's keys in physical page 0
    auto load_tile = [&](int tile0) {       // (positions beyond the block's reach repeat the last one: finite, and masked below)
#pragma unroll
        for (int i = 0; i < CH; i++) {
            const int pc = t + NT * i, pos = pc / (HD / 8), dq = pc % (HD / 8);
            const int ap = min(tile0 + pos, last_pos);
            kreg[i] = *(const u32x4_t *)(kv_head + (size_t)pages[ap >> a.logP] * page_stride + ((ap & (P - 1)) * HD + 8 * dq));
        }
        {
            const int ap = min(tile0 + (t & 127), last_pos);                // one position per thread, CH chunks of it
            const kvhalf_t *Vp = kv_head + (size_t)pages[ap >> a.logP] * page_stride + ((P + (ap & (P - 1))) * HD + 8 * (t >> 7));
#pragma unroll
            for (int i = 0; i < CH; i++) vreg[i] = *(const u32x4_t *)(Vp + 8 * VSTEP * i);
        }
    };
    load_tile(0);                               // under the preparation of the queries

    // queries: rotate, scale, split into half hi + lo, in B-operand order (8 consecutive dimensions per lane and step)
    f16x8_t qhi[KS], qlo[KS];
    {
        const float *q = a.qkv + (size_t)min(row, a.T - 1) * 3 * d + h * HD;
        const float2 *rp = a.rope + (size_t)min(qpos, a.pos0 + a.T - 1) * HH;
        const float qscale = rsqrtf((float)HD);
        // all loads first (8 consecutive dimensions: 16-byte loads), then the arithmetic
        float4 x0v[KS][2], x1v[KS][2], csv[KS][4];
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            const int i0 = (32 * ks + 8 * g) % HH;
#pragma unroll
            for (int j = 0; j < 2; j++) {
                x0v[ks][j] = *(const float4 *)(q + i0 + 4 * j);
                x1v[ks][j] = *(const float4 *)(q + i0 + HH + 4 * j);
            }
#pragma unroll
            for (int j = 0; j < 4; j++) csv[ks][j] = *(const float4 *)(rp + i0 + 2 * j);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            const float x0a[8] = {x0v[ks][0].x, x0v[ks][0].y, x0v[ks][0].z, x0v[ks][0].w, x0v[ks][1].x, x0v[ks][1].y, x0v[ks][1].z, x0v[ks][1].w};
            const float x1a[8] = {x1v[ks][0].x, x1v[ks][0].y, x1v[ks][0].z, x1v[ks][0].w, x1v[ks][1].x, x1v[ks][1].y, x1v[ks][1].z, x1v[ks][1].w};
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const int dim = 32 * ks + 8 * g + e;
                const float4 c4 = csv[ks][e >> 1];
                const float2 cs = (e & 1) ? make_float2(c4.z, c4.w) : make_float2(c4.x, c4.y);
                const float v = rounded((dim < HH ? rot_lo(x0a[e], x1a[e], cs) : rot_hi(x0a[e], x1a[e], cs)) * qscale);
                const _Float16 hi = (_Float16)v;
                qhi[ks][e] = hi;
                qlo[ks][e] = (_Float16)(v - (float)hi);
            }
        }
    }
    f32x4_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;       // running maximum of the row (same in its four lanes), this lane's share of the sum

    // column of position pos inside a dimension row of V^T: [u = pos / 32][g = (pos % 16) / 4][j = 4 ((pos / 16) % 2) + pos % 4]
    uint16_t *vt_lane;
    uint32_t vt_sel;
    {
        const int pos = t & 127, odd = pos & 1;
        const int col = (pos >> 5) * 32 + ((pos & 15) >> 2) * 8 + ((pos >> 4) & 1) * 4 + (pos & 3);
        vt_lane = &Vt[0][(8 * (t >> 7) + odd) * VROW + (col & ~1)];
        vt_sel = odd ? 0x03020706u : 0x05040100u;   // (hi of other, hi of mine) : (lo of mine, lo of other)
    }
    const int wave_first = a.pos0 + rb * ROWS + wave * 16;        // position of the wave's first row
    // tile in registers -> LDS buffer bf: keys as stored; values transposed: a 32-bit word of the thread holds
    // dimensions (2 j, 2 j + 1) of its position; with the neighbouring lane's word (position ^ 1) the even lane
    // forms the pair of positions of dimension 2 j and the odd lane that of dimension 2 j + 1: one byte
    // permutation and one 32-bit LDS write per word
    auto write_tile = [&](int bf) {
#pragma unroll
        for (int i = 0; i < CH; i++) {
            const int pc = t + NT * i, pos = pc / (HD / 8), dq = pc % (HD / 8);
            *(u32x4_t *)&Ks[bf][pos * KROW + 8 * dq] = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < CH; i++) {
#pragma unroll
            for (int w = 0; w < 4; w++) {
                const uint32_t mine = vreg[i][w];
                const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0xB1, 0xF, 0xF, false);   // lane ^ 1
                *(uint32_t *)(vt_lane + bf * (HD * VROW) + (8 * VSTEP * i + 2 * w) * VROW) = __builtin_amdgcn_perm(other, mine, vt_sel);
            }
        }
    };
    // One tile in LDS: barrier, write, barrier, then the next tile's loads fly under this tile's multiplications.
    // Two tiles in LDS: the next tile is written into the other buffer after this tile's multiplications (no wave
    // reads that buffer any more: its tile was finished before the last barrier), one barrier per tile.
    if (NBUF == 2) {
        write_tile(0);
        __syncthreads();
    }
    for (int kt = 0; kt < n_tiles; kt++) {
        const int tile0 = kt << 7, bf = NBUF == 2 ? (kt & 1) : 0;
        const bool more = kt + 1 < n_tiles;
        if (NBUF == 1) {
            __syncthreads();                    // the previous tile has been consumed
            write_tile(0);
            __syncthreads();
        }
        if (more) load_tile(tile0 + 128);
        if (tile0 <= wave_last) {               // else nothing of this tile is visible to the wave's rows (uniform in the wave)
            // scores of 128 positions x 16 query rows
            f32x4_t s[8];
#pragma unroll
            for (int pt = 0; pt < 8; pt++) {
                s[pt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ks++) {
                    const f16x8_t kk = __builtin_bit_cast(f16x8_t, *(const u32x4_t *)&Ks[bf][(16 * pt + q16) * KROW + 32 * ks + 8 * g]);
                    s[pt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kk, qhi[ks], s[pt], 0, 0, 0);
                    s[pt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kk, qlo[ks], s[pt], 0, 0, 0);
                }
            }
            // causal mask (only a tile that reaches beyond the wave's first row needs it), tile maximum of the row.
            // Every row sees position 0, so its maximum is finite from the first tile on; rows beyond the pass are
            // computed like the others (on the last row's queries) and dropped.
            if (tile0 + 127 > wave_first) {
#pragma unroll
                for (int pt = 0; pt < 8; pt++)
#pragma unroll
                    for (int r = 0; r < 4; r++)
                        s[pt][r] = (tile0 + 16 * pt + 4 * g + r <= qpos) ? s[pt][r] : -INFINITY;
            }
            float mx = -INFINITY;
#pragma unroll
            for (int pt = 0; pt < 8; pt++)
#pragma unroll
                for (int r = 0; r < 4; r++) mx = fmaxf(mx, s[pt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float scale = __expf(m_run - m_new);              // 0 in the first tile (m_run = -inf)
            float psum = 0.f;
            f16x8_t pa[4];
#pragma unroll
            for (int pt = 0; pt < 8; pt++)
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const float p = __expf(s[pt][r] - m_new);       // 0 for a masked score
                    psum += p;
                    pa[pt >> 1][4 * (pt & 1) + r] = (_Float16)p;
                }
            l_run = l_run * scale + psum;
            m_run = m_new;
            // rescale the output rows 4 g + r by the factor of their query row, then add P.V
            float sc[4];
#pragma unroll
            for (int r = 0; r < 4; r++) sc[r] = __shfl(scale, 4 * g + r);
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
#pragma unroll
                for (int r = 0; r < 4; r++) o[dt][r] *= sc[r];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const f16x8_t vv = __builtin_bit_cast(f16x8_t, *(const u32x4_t *)&Vt[bf][(16 * dt + q16) * VROW + 32 * u + 8 * g]);
                    o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa[u], vv, o[dt], 0, 0, 0);
                }
            }
        }
        if (NBUF == 2) {
            if (more) write_tile(bf ^ 1);
            __syncthreads();
        }
    }
    // normalise and store: lane holds dimension 16 dt + q16 of query rows 4 g + r
    float l = l_run + __shfl_xor(l_run, 16);
    l += __shfl_xor(l, 32);
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const float ir = __shfl(inv, 4 * g + r);
        const int orow = rb * ROWS + wave * 16 + 4 * g + r;
        if (orow < a.T) {
#pragma unroll
            for (int dt = 0; dt < DT; dt++)
                store_act_pf(a.act_out, a.act_blk_bytes, orow >> 3, orow & 7, h * HD + 16 * dt + q16, o[dt][r] * ir, a.act_pair);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Random numbers of sampling mode: Philox4x32-10 (Salmon et al., SC 2011), a counter-based generator,
// so that the number for (absolute token position, purpose) can be produced by whichever kernel
// needs it, with no state to carry and independent of the control flow that led there.
// Ten rounds on the counter words (c0, c1, c2, c3) under the key (k0, k1):
//   (c0, c1, c2, c3) <- (mulhi(B, c2) ^ c1 ^ k0, B * c2, mulhi(A, c0) ^ c3 ^ k1, A * c0),
// A = 0xD2511F53, B = 0xCD9E8D57, products mod 2^32; the key grows by (0x9E3779B9, 0xBB67AE85)
// between rounds.  Returns the first word of the block for counter (position, purpose, 0, 0).
__device__ __forceinline__ uint32_t philox_word(uint32_t k0, uint32_t k1, uint32_t position, uint32_t purpose)
{
    uint32_t a = position, b = purpose, c = 0u, d = 0u;
#pragma unroll
    for (int r = 0; r < 10; r++) {
        const uint32_t ha = __umulhi(0xD2511F53u, a), la = 0xD2511F53u * a;
        const uint32_t hc = __umulhi(0xCD9E8D57u, c), lc = 0xCD9E8D57u * c;
        a = hc ^ b ^ (k0 + (uint32_t)r * 0x9E3779B9u);
        c = ha ^ d ^ (k1 + (uint32_t)r * 0xBB67AE85u);
        b = lc;
        d = la;
    }
    return a;
}
// uniform number in [0, 1) with 24 random bits
__device__ __forceinline__ float philox_uniform(uint32_t k0, uint32_t k1, uint32_t position, uint32_t purpose)
{
    return (float)(philox_word(k0, k1, position, purpose) >> 8) * (1.f / 16777216.f);
}

__global__ void philox_words_kernel(uint32_t k0, uint32_t k1, uint32_t pos0, uint32_t purpose, int n, uint32_t *out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = philox_word(k0, k1, pos0 + (uint32_t)i, purpose);
}

// Where the uniform numbers of a launch's rows come from: the generator keyed by the seed, evaluated
// at the absolute position each row decides, or numbers the caller supplied (a test hook).
struct USrc {
    int from_seed;
    uint32_t k0, k1;
    int pos[KG_ROWS];
    float u0[KG_ROWS], u1[KG_ROWS];     // caller's numbers for the launch's first / second purpose
};
__device__ __forceinline__ float row_uniform(const USrc &s, int row, int purpose, int which)
{
    // constant indices only: the argument block stays in scalar registers
    float tv = 0.f;
    int pv = 0;
#pragma unroll
    for (int i = 0; i < KG_ROWS; i++)
        if (i == row) { tv = which ? s.u1[i] : s.u0[i]; pv = s.pos[i]; }
    return s.from_seed ? philox_uniform(s.k0, s.k1, (uint32_t)pv, (uint32_t)purpose) : tv;
}

// ---------------------------------------------------------------------------------------------
// Block-wide inverse-CDF draw (1024 threads): smallest index n with w(0) + .. + w(n) > u * total,
// walking ascending indices; weights are accumulated in double.  Returns -1 when total == 0.
// All threads must call it; all get the result.  The weight of index i is w(za[i], zb[i]) (zb may be
// null: its value is then 0).
// Up to 32768 indices every thread owns 32 consecutive ones: it fetches them with 16-byte loads,
// computes their weights once and keeps them in registers for the sum, the walk and the fallback;
// larger index sets are walked in chunks with the weights recomputed.
struct I8 { int v[KG_ROWS]; };

template <class F>
__device__ int block_inverse_cdf(const float *za, const float *zb, F w, int V, float u)
{
    __shared__ double wsum[16];
    __shared__ int found, lastpos;
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const bool in_regs = V <= 32768 && (V & 3) == 0;
    const int chunk = in_regs ? 32 : (V + 1023) >> 10;
    const int i0 = min(V, t * chunk), i1 = min(V, i0 + chunk);
    float wv[32];
    double local = 0.0;
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < 32; j += 4) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            const bool in = i0 + j < i1;                       // V % 4 == 0: a group of four is all in or all out
            if (in) {
                a = *(const float4 *)(za + i0 + j);
                if (zb) b = *(const float4 *)(zb + i0 + j);
            }
            wv[j] = in ? w(a.x, b.x) : 0.f;
            wv[j + 1] = in ? w(a.y, b.y) : 0.f;
            wv[j + 2] = in ? w(a.z, b.z) : 0.f;
            wv[j + 3] = in ? w(a.w, b.w) : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 32; j++) local += (double)wv[j];
    } else {
        for (int i = i0; i < i1; i++) local += (double)w(za[i], zb ? zb[i] : 0.f);
    }
    double incl = local;                                   // inclusive scan inside the wave
    for (int o = 1; o < 64; o <<= 1) {
        double v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    if (t == 0) { found = -1; lastpos = -1; }
    __syncthreads();
    double base = 0.0, total = 0.0;
    for (int k = 0; k < 16; k++) {
        if (k < wave) base += wsum[k];
        total += wsum[k];
    }
    if (total <= 0.0) return -1;
    const double thr = (double)u * total;
    const double excl = base + incl - local;
    if (excl <= thr && excl + local > thr) {
        double acc = excl;
        if (in_regs) {
            int f = -1;
#pragma unroll
            for (int j = 0; j < 32; j++) {
                acc += (double)wv[j];
                if (f < 0 && acc > thr) f = i0 + j;
            }
            if (f >= 0) found = f;
        } else {
            for (int i = i0; i < i1; i++) {
                acc += (double)w(za[i], zb ? zb[i] : 0.f);
                if (acc > thr) { found = i; break; }
            }
        }
    }
    __syncthreads();
    if (found >= 0) return found;
    // u * total landed beyond the accumulated mass by rounding: last index with weight
    int lp = -1;
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < 32; j++) if (wv[j] > 0.f) lp = i0 + j;
    } else {
        for (int i = i0; i < i1; i++) if (w(za[i], zb ? zb[i] : 0.f) > 0.f) lp = i;
    }
    if (lp >= 0) atomicMax(&lastpos, lp);
    __syncthreads();
    return lastpos;
}

// Block-wide inverse-CDF draw from softmax(z / T) through the LM head's per-tile statistics (1024
// threads): tile i (16 consecutive tokens) weighs s_i exp(m_i - mx), so the tile that holds u * total is
// found from n_tiles numbers, and only its 16 logits are looked at.  Walks ascending token indices;
// sums in double.  Returns -1 when the total is not positive.  All threads must call it; all get the result.
// hs: statistics of the row, tile i at hs[4 i] = (max of z / T, sum exp(z / T - max), ..).
__device__ int tile_inverse_cdf(const float *hs, int n_tiles, const float *z, float inv_temp, float mx, float u)
{
    __shared__ double wsum[16];
    __shared__ int cand[16];
    __shared__ int found;
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int chunk = (n_tiles + 1023) >> 10;
    const int i0 = min(n_tiles, t * chunk), i1 = min(n_tiles, i0 + chunk);
    auto weight = [&](int i) {
        const float2 ms = *(const float2 *)(hs + (size_t)i * 4);
        return (double)(ms.y * __expf(ms.x - mx));
    };
    double local = 0.0;
    for (int i = i0; i < i1; i++) local += weight(i);
    double incl = local;                                   // inclusive scan inside the wave
    for (int o = 1; o < 64; o <<= 1) {
        double v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    if (t == 0) found = -1;
    __syncthreads();
    double base = 0.0, total = 0.0;
    for (int k = 0; k < 16; k++) {
        if (k < wave) base += wsum[k];
        total += wsum[k];
    }
    if (!(total > 0.0)) return -1;
    const double thr = (double)u * total;                  // u < 1: below the total
    const double excl = base + incl - local;
    // the stretch that holds the threshold: the last one that starts at or below it
    const unsigned long long starts_below = __ballot(i0 < i1 && excl <= thr);
    if (lane == 0) cand[wave] = starts_below ? wave * 64 + 63 - __builtin_clzll(starts_below) : -1;
    __syncthreads();
    int owner = -1;
    for (int k = 0; k < 16; k++) owner = max(owner, cand[k]);
    if (t == owner) {
        double acc = excl;
        int tile = -1;
        for (int i = i0; i < i1; i++) {
            const double wt = weight(i);
            if (wt > 0.0) {
                if (tile >= 0) acc += weight(tile);        // pass the tile before: the threshold lies beyond it
                tile = i;
                if (acc + wt > thr) break;
            }
        }
        // (a stretch whose sums fall short of the threshold by rounding ends at its last tile with weight)
        if (tile >= 0) {
            // inside the tile the 16 weights are recomputed; if their sum misses the tile's own by rounding,
            // the tile's last token with weight is the draw
            int f = -1, lastw = -1;
            for (int j = 0; j < 16; j++) {
                const float wj = __expf(z[tile * 16 + j] * inv_temp - mx);
                acc += (double)wj;
                if (wj > 0.f) lastw = tile * 16 + j;
                if (f < 0 && acc > thr) f = tile * 16 + j;
            }
            found = f >= 0 ? f : lastw;
        }
    }
    __syncthreads();
    return found;
}

// Final reduction of the per-tile LM-head statistics for one row per block: arg-max (lowest index
// among equal maxima) and top-1 probability of softmax(z / T) = 1 / sum exp((z - max) / T).
// mode 1 additionally draws the token from softmax(z / T) with the row's uniform number (of the
// given purpose: 0 a draft token, 2 a first / plain token).
// stat_out[row] = (max of z/T, sum exp(z/T - max)).
__global__ __launch_bounds__(1024) void head_final_kernel(const float *hstat, int n_tiles, const float *logits,
                                                          int V, float inv_temp, int mode, USrc us, int purpose, int *tok_out,
                                                          float *conf_out, float *stat_out)
{
    __shared__ float bm[16], bs[16];
    __shared__ int bi[16];
    __shared__ float fin[2];
    __shared__ int fin_i;
    const int m = blockIdx.x, t = threadIdx.x, wave = t >> 6, lane = t & 63;
    float best = -INFINITY, sum = 0.f;
    int idx = 0x7FFFFFFF;
    for (int i = t; i < n_tiles; i += 1024) {
        const float4 hs = *(const float4 *)(hstat + ((size_t)m * n_tiles + i) * 4);
        float mx = hs.x, sm = hs.y;
        int id = __float_as_int(hs.z);
        if (mx > best) { sum = sum * __expf(best - mx) + sm; best = mx; idx = id; }
        else { sum += sm * __expf(mx - best); if (mx == best && id < idx) idx = id; }
    }
    for (int o = 32; o >= 1; o >>= 1) {
        float om = __shfl_xor(best, o), os = __shfl_xor(sum, o);
        int oi = __shfl_xor(idx, o);
        float nm = fmaxf(best, om);
        float a = (best == -INFINITY) ? 0.f : sum * __expf(best - nm);
        float b = (om == -INFINITY) ? 0.f : os * __expf(om - nm);
        if (om > best || (om == best && oi < idx)) idx = oi;
        best = nm;
        sum = a + b;
    }
    if (lane == 0) { bm[wave] = best; bs[wave] = sum; bi[wave] = idx; }
    __syncthreads();
    if (t == 0) {
        best = bm[0]; sum = bs[0]; idx = bi[0];
        for (int w = 1; w < 16; w++) {
            float nm = fmaxf(best, bm[w]);
            float a = (best == -INFINITY) ? 0.f : sum * __expf(best - nm);
            float b = (bm[w] == -INFINITY) ? 0.f : bs[w] * __expf(bm[w] - nm);
            if (bm[w] > best || (bm[w] == best && bi[w] < idx)) idx = bi[w];
            best = nm;
            sum = a + b;
        }
        fin[0] = best; fin[1] = sum; fin_i = idx;
        conf_out[m] = 1.f / sum;
        stat_out[2 * m] = best;
        stat_out[2 * m + 1] = sum;
        if (mode == 0) tok_out[m] = idx;
    }
    if (mode == 0) return;
    __syncthreads();
    const int tok = tile_inverse_cdf(hstat + (size_t)m * n_tiles * 4, n_tiles, logits + (size_t)m * V, inv_temp, fin[0],
                                     row_uniform(us, m, purpose, 0));
    if (t == 0) tok_out[m] = tok < 0 ? fin_i : tok;
}

// Speculative-sampling acceptance of one round (Section 3: the first rejected draft discards the
// rest; the sampling distribution of the target is preserved).  Draft d_i ~ q_i is kept while
// u_acc[i] < min(1, p_i(d_i) / q_i(d_i)); the first rejected position is redrawn from
// normalize(max(0, p_i - q_i)); if all k are kept a bonus token is drawn from p_k.
// Row i decides the token at us.pos[i]; its acceptance number has purpose 1 (us.u0), its redraw /
// bonus number purpose 2 (us.u1).
// zt: target logits [k+1][V], zd: draft logits [k][V]; tstat/dstat: (max, sum exp) per row of z/T.
// out[0] = number of accepted drafts, out[1] = the redrawn / bonus token.
__global__ __launch_bounds__(1024) void accept_sample_kernel(const float *zt, const float *zd, const float *tstat,
                                                             const float *dstat, const float *hstat_t, int V, int k,
                                                             float inv_temp, I8 drafts, USrc us, int *out)
{
    __shared__ int n_acc;
    const int t = threadIdx.x;
    // the k acceptance tests are independent: lane n tests draft n, the first failure ends the run
    if (t < 64) {
        bool keep = true;
        if (t < k) {
            int dd = 0;
#pragma unroll
            for (int i = 0; i < KG_ROWS; i++)
                if (i == t) dd = drafts.v[i];
            const float pp = __expf(zt[(size_t)t * V + dd] * inv_temp - tstat[2 * t]) / tstat[2 * t + 1];
            const float qq = __expf(zd[(size_t)t * V + dd] * inv_temp - dstat[2 * t]) / dstat[2 * t + 1];
            float uv = 0.f;
#pragma unroll
            for (int i = 0; i < KG_ROWS; i++)
                if (i == t) uv = row_uniform(us, i, 1, 0);
            keep = uv < fminf(1.f, pp / qq);
        }
        const unsigned long long rejected = __ballot(!keep);
        if (t == 0) n_acc = rejected ? min(k, __builtin_ctzll(rejected)) : k;
    }
    __syncthreads();
    const int n = n_acc;
    const float *zp = zt + (size_t)n * V;
    const float pm = tstat[2 * n], ps = 1.f / tstat[2 * n + 1];
    int tok = -1;
    if (n < k) {
        const float *zq = zd + (size_t)n * V;
        const float qm = dstat[2 * n], qs = 1.f / dstat[2 * n + 1];
        tok = block_inverse_cdf(
            zp, zq, [&](float a, float b) { return fmaxf(0.f, __expf(a * inv_temp - pm) * ps - __expf(b * inv_temp - qm) * qs); }, V,
            row_uniform(us, n, 2, 1));
        __syncthreads();
    }
    // all drafts kept (or an empty residual): the bonus token from p_n, through the target head's tile statistics
    if (tok < 0) tok = tile_inverse_cdf(hstat_t + (size_t)n * (V / 16) * 4, V / 16, zp, inv_temp, pm, row_uniform(us, n, 2, 1));
    if (t == 0) { out[0] = n; out[1] = tok; }
}

// Streaming read of a buffer with no dependencies between the loads: the bandwidth that a weight
// stream could reach at best on this device (the measured ceiling the projections are compared
// with).  Persistent grid, 8 x 16-byte loads in flight per lane; out[block] keeps the loads alive.
__global__ __launch_bounds__(512, 2) void stream_read_kernel(const u32x4_t *__restrict__ src, size_t n16, unsigned *out)
{
    // a block takes 64 KB pieces; inside a piece every wave reads 8 consecutive KB (as a wave of a
    // projection reads consecutive 1 KB weight tiles)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t pieces = (n16 + 4095) >> 12;
    unsigned x = 0;
    for (size_t pc = blockIdx.x; pc < pieces; pc += gridDim.x) {
        const size_t base = (pc << 12) + (size_t)wave * 512 + lane;
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const size_t i = base + (size_t)u * 64;
            v[u] = i < n16 ? __builtin_nontemporal_load(src + i) : u32x4_t{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 8; u++) x ^= v[u][0] ^ v[u][3];
    }
    for (int o = 32; o >= 1; o >>= 1) x ^= __shfl_xor(x, o);
    if (lane == 0) atomicXor(&out[blockIdx.x], x);
}

// Zero n16 16-byte pieces (a launch that a stream capture can record, unlike a memset node).
__global__ void fill_zero_kernel(u32x4_t *p, unsigned n16)
{
    const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n16) p[i] = u32x4_t{0u, 0u, 0u, 0u};
}

// Copy cached k and v rows of one position, widened to float (test / debug access).
template <typename T>
__global__ void kv_read_kernel(const void *kv, const int *page_table, int slot, int n_slots, int H, int hd,
                               int P, int logP, int pos, float *k_out, float *v_out)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= H * hd) return;
    int h = i / hd, e = i % hd;
    const T *Kp = (const T *)kv + ((((size_t)page_table[pos >> logP] * n_slots + slot) * H + h) * 2) * (size_t)P * hd;
    int pl = pos & (P - 1);
    k_out[i] = kv_ld<T>(Kp + (size_t)pl * hd + e);
    v_out[i] = kv_ld<T>(Kp + (size_t)P * hd + (size_t)pl * hd + e);
}
