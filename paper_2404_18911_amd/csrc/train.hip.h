// Device code of the adapter's training step (Section 3.1, "Training Loss", Eq. 3; AdamW per
// Section 4.1): the adapter runs over all T positions of a sequence at once, the cross entropy of
// its draft distribution against the frozen target's is differentiated by hand (chain rule written
// out: RMSNorm, rotary embedding, causal attention, projections), and AdamW updates fp32 master
// copies of the adapter's tensors.  All arithmetic is fp32; the dense contractions go through the
// fp32 MFMA (32x32x2), weights of the frozen LM head are read from their bf16 tiles and widened
// exactly.  Included by kangaroo.hip after kernels.hip.h.
#pragma once

typedef float f32x16_t __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------------------
// C[M][N] (+)= sum_k A(m, k) * B(k, n), fp32, any strides.
//   A(m, k) = A[m * sam + k * sak]
//   B(k, n) = b_mode 0: B[k * sbk + n * sbn]
//             b_mode 1: element (row n, col k) of a matrix stored as bf16 MFMA tiles (the layout of
//                       pack_w_bf16_kernel: tile (row/16, col/32), 16-byte unit (col%32/8)*16 + row%16)
//             b_mode 2: element (row k, col n) of such a matrix
// One workgroup (4 waves) per 64 x 128 tile of C; a wave owns 32 x 64 of it (two 32x32x2 MFMA tiles
// that share the A operand).  k advances in steps of 16 through two LDS buffers: the next step's
// operands are fetched into registers while the current one is multiplied, and stored to the other
// buffer afterwards, so a step has one barrier.  A thread fetches 4 consecutive elements of A and
// 2 x 4 of B along whichever index is contiguous in memory (one 16-byte load when the host found
// the operand aligned for it: a_vec / b_vec), with element-wise guards at the ragged edges.
// A contraction with few output tiles and a long k is split over blockIdx.z: slice z handles k in
// [z * k_chunk, (z + 1) * k_chunk) and writes its own partial [M][N] at part + z * M * N; a second
// kernel adds the slices in order (no atomics: the result does not depend on scheduling).
// With batch > 1 the launch holds one product per blockIdx.z instead (the per-head products of the
// attention: operands and result advance by bsa / bsb / bsc elements per head).
struct TrGemm {
    const void *A; long sam, sak;
    const void *B; long sbk, sbn;
    int b_mode, b_KS;
    float *C; long ldc;
    int M, N, K;
    int accumulate;
    int k_chunk;        // k handled per blockIdx.z slice (a multiple of 16); >= K when not split
    float *part;        // partial results of a split contraction
    int a_vec, b_vec;   // 4 consecutive elements along the contiguous index are one aligned 16-byte word
    int batch;          // > 1: blockIdx.z is a batch index (one product per attention head), k is not split
    long bsa, bsb, bsc; // element offsets of A, B (b_mode 0) and C per batch index
};

// LDS row strides in floats.  A thread stores its 4 fetched elements either down 4 consecutive rows
// (operand contiguous along k: the lanes of a wave then cover rows 4 apart) or as one 16-byte word
// (operand contiguous along m / n).  With 4 * stride = 16 (mod 64) the first pattern spreads over all
// banks; strides are multiples of 4 floats so that the 16-byte stores are aligned.
#ifndef TRG_LDA
#define TRG_LDA 100
#define TRG_LDB 164
#endif

__device__ __forceinline__ size_t packed_u16_index(int row, int col, int KS)
{
    return ((((size_t)(row >> 4) * KS + tile_pos(col >> 5, KS)) * 64 + ((col >> 3) & 3) * 16 + (row & 15)) << 3) + (col & 7);
}

__global__ __launch_bounds__(256) void tr_gemm_kernel(const TrGemm g)
{
    __shared__ __attribute__((aligned(16))) float As[2][16][TRG_LDA];
    __shared__ __attribute__((aligned(16))) float Bs[2][16][TRG_LDB];
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 128;
    const int wm = (wave & 1) * 32, wn = (wave >> 1) * 64;
    const bool a_kc = g.sak == 1;                      // A contiguous along k
    const bool b_kc = g.b_mode == 0 ? g.sbk == 1 : g.b_mode == 1;
    const bool batched = g.batch > 1;
    const bool split = !batched && gridDim.z > 1;
    const int k_lo = batched ? 0 : blockIdx.z * g.k_chunk, k_hi = batched ? g.K : min(g.K, k_lo + g.k_chunk);
    const size_t boa = batched ? (size_t)blockIdx.z * g.bsa : 0, bob = batched ? (size_t)blockIdx.z * g.bsb : 0,
                 boc = batched ? (size_t)blockIdx.z * g.bsc : 0;
    // first of the 4 (A) and 2 x 4 (B, second group 64 columns further) elements this thread fetches per step
    int am, ak, bn, bk;
    if (a_kc) { am = t >> 2; ak = (t & 3) * 4; } else { ak = t >> 4; am = (t & 15) * 4; }
    if (b_kc) { bn = t >> 2; bk = (t & 3) * 4; } else { bk = t >> 4; bn = (t & 15) * 4; }
    const float *pa = (const float *)g.A + boa + (size_t)(m0 + am) * g.sam + (size_t)(k_lo + ak) * g.sak;
    const long a_step = 16 * g.sak, a_el = a_kc ? g.sak : g.sam;
    const float *pb0 = nullptr, *pb1 = nullptr;        // b_mode 0
    long b_step = 0, b_el = 0;
    const uint16_t *Bp = (const uint16_t *)g.B;        // tiled modes
    size_t rb0 = 0, rb1 = 0;                           // mode 1: per-row part of the tile index; mode 2: full index at k_lo
    if (g.b_mode == 0) {
        pb0 = (const float *)g.B + bob + (size_t)(k_lo + bk) * g.sbk + (size_t)(n0 + bn) * g.sbn;
        pb1 = pb0 + (size_t)64 * g.sbn;
        b_step = 16 * g.sbk;
        b_el = b_kc ? g.sbk : g.sbn;
    } else if (g.b_mode == 1) {
        rb0 = (size_t)((n0 + bn) >> 4) * g.b_KS * 64 + ((n0 + bn) & 15);
        rb1 = (size_t)((n0 + bn + 64) >> 4) * g.b_KS * 64 + ((n0 + bn + 64) & 15);
    } else {
        rb0 = packed_u16_index(k_lo + bk, n0 + bn, g.b_KS);
        rb1 = packed_u16_index(k_lo + bk, n0 + bn + 64, g.b_KS);
    }
    const bool am_all = a_kc ? (m0 + am < g.M) : (m0 + am + 3 < g.M);
    float av[4], bv[2][4];
    auto widen = [](uint2 raw, float *o) {
        o[0] = __uint_as_float(raw.x << 16);
        o[1] = __uint_as_float(raw.x & 0xFFFF0000u);
        o[2] = __uint_as_float(raw.y << 16);
        o[3] = __uint_as_float(raw.y & 0xFFFF0000u);
    };
    auto fetch = [&](int k0) {
        // ---- A
        const bool ak_all = a_kc ? (k0 + ak + 3 < k_hi) : (k0 + ak < k_hi);
        if (g.a_vec && am_all && ak_all) {
            const float4 v = *(const float4 *)pa;
            av[0] = v.x; av[1] = v.y; av[2] = v.z; av[3] = v.w;
        } else {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int m = m0 + am + (a_kc ? 0 : i), k = k0 + ak + (a_kc ? i : 0);
                av[i] = (m < g.M && k < k_hi) ? pa[i * a_el] : 0.f;
            }
        }
        pa += a_step;
        // ---- B
        if (g.b_mode == 0) {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const float *pb = h ? pb1 : pb0;
                const int nb = n0 + bn + 64 * h;
                const bool n_all = b_kc ? (nb < g.N) : (nb + 3 < g.N);
                const bool k_all = b_kc ? (k0 + bk + 3 < k_hi) : (k0 + bk < k_hi);
                if (g.b_vec && n_all && k_all) {
                    const float4 v = *(const float4 *)pb;
                    bv[h][0] = v.x; bv[h][1] = v.y; bv[h][2] = v.z; bv[h][3] = v.w;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const int n = nb + (b_kc ? 0 : i), k = k0 + bk + (b_kc ? i : 0);
                        bv[h][i] = (n < g.N && k < k_hi) ? pb[i * b_el] : 0.f;
                    }
                }
            }
            pb0 += b_step;
            pb1 += b_step;
        } else if (g.b_mode == 1) {
            // four consecutive columns (k) of rows n, n + 64 of the tiled matrix: 8 bytes each, 8-byte aligned;
            // N, K and k_chunk are multiples of 8, so the four share the bounds verdict
            const int col = k0 + bk;
            const size_t cpart = (size_t)tile_pos(col >> 5, g.b_KS) * 64 + ((col >> 3) & 3) * 16;
            const bool k_ok = col < k_hi;
            uint2 r0 = make_uint2(0u, 0u), r1 = make_uint2(0u, 0u);
            if (k_ok && n0 + bn < g.N) r0 = *(const uint2 *)(Bp + ((rb0 + cpart) << 3) + (col & 7));
            if (k_ok && n0 + bn + 64 < g.N) r1 = *(const uint2 *)(Bp + ((rb1 + cpart) << 3) + (col & 7));
            widen(r0, bv[0]);
            widen(r1, bv[1]);
        } else {
            // four consecutive columns (n) of row k: the row advances by 16 per step, i.e. by one tile row
            const bool k_ok = k0 + bk < k_hi;
            uint2 r0 = make_uint2(0u, 0u), r1 = make_uint2(0u, 0u);
            if (k_ok && n0 + bn < g.N) r0 = *(const uint2 *)(Bp + rb0);
            if (k_ok && n0 + bn + 64 < g.N) r1 = *(const uint2 *)(Bp + rb1);
            widen(r0, bv[0]);
            widen(r1, bv[1]);
            rb0 += (size_t)g.b_KS * 512;
            rb1 += (size_t)g.b_KS * 512;
        }
    };
    auto stash = [&](int buf) {
        if (a_kc) {
#pragma unroll
            for (int i = 0; i < 4; i++) As[buf][ak + i][am] = av[i];
        } else {
            *(float4 *)&As[buf][ak][am] = make_float4(av[0], av[1], av[2], av[3]);
        }
#pragma unroll
        for (int h = 0; h < 2; h++) {
            if (b_kc) {
#pragma unroll
                for (int i = 0; i < 4; i++) Bs[buf][bk + i][bn + 64 * h] = bv[h][i];
            } else {
                *(float4 *)&Bs[buf][bk][bn + 64 * h] = make_float4(bv[h][0], bv[h][1], bv[h][2], bv[h][3]);
            }
        }
    };
    f32x16_t acc0, acc1;
#pragma unroll
    for (int i = 0; i < 16; i++) { acc0[i] = 0.f; acc1[i] = 0.f; }
    int buf = 0;
    if (k_lo < k_hi) {
        fetch(k_lo);
        stash(0);
    }
    __syncthreads();
    for (int k0 = k_lo; k0 < k_hi; k0 += 16) {
        const bool more = k0 + 16 < k_hi;
        if (more) fetch(k0 + 16);                       // in flight while this step is multiplied
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
            const float a = As[buf][2 * kk + (lane >> 5)][wm + (lane & 31)];
            const float b0 = Bs[buf][2 * kk + (lane >> 5)][wn + (lane & 31)];
            const float b1 = Bs[buf][2 * kk + (lane >> 5)][wn + 32 + (lane & 31)];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc1, 0, 0, 0);
        }
        if (more) stash(buf ^ 1);                       // the other buffer was last read before the previous barrier
        __syncthreads();
        buf ^= 1;
    }
    // accumulator register i of lane l: row 8 * (i / 4) + 4 * (l / 32) + i % 4, column l % 32
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const int n = n0 + wn + 32 * h + (lane & 31);
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int m = m0 + wm + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
            const float v = h ? acc1[i] : acc0[i];
            if (m < g.M && n < g.N) {
                if (split) {
                    g.part[((size_t)blockIdx.z * g.M + m) * g.N + n] = v;
                } else {
                    float *c = g.C + boc + (size_t)m * g.ldc + n;
                    *c = g.accumulate ? *c + v : v;
                }
            }
        }
    }
}

// C[m][n] (+)= part[0][m][n] + part[1][m][n] + ... in slice order
__global__ void tr_gemm_reduce_kernel(const float *part, int S, int M, int N, float *C, long ldc, int accumulate)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)M * N) return;
    float s = part[i];
    for (int z = 1; z < S; z++) s += part[(size_t)z * M * N + i];
    float *c = C + (i / N) * ldc + (i % N);
    *c = accumulate ? *c + s : s;
}

// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float tr_block_sum(float v, float *red)
{
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float s = 0.f;
    for (int w = 0; w < nw; w++) s += red[w];
    return s;
}
__device__ __forceinline__ float tr_block_max(float v, float *red)
{
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    float s = red[0];
    for (int w = 1; w < nw; w++) s = fmaxf(s, red[w]);
    return s;
}

// y[t] = x[t] * r[t] * g with r[t] = rsqrt(mean(x[t]^2) + eps); one block per row
__global__ __launch_bounds__(256) void tr_rmsnorm_kernel(const float *x, const float *g, int d, float eps, float *y, float *r)
{
    __shared__ float red[4];
    const int row = blockIdx.x;
    const float *xr = x + (size_t)row * d;
    float s = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) s += xr[i] * xr[i];
    s = tr_block_sum(s, red);
    const float rr = 1.f / sqrtf(s / (float)d + eps);
    if (threadIdx.x == 0) r[row] = rr;
    for (int i = threadIdx.x; i < d; i += 256) y[(size_t)row * d + i] = xr[i] * rr * g[i];
}

// dx[t] = r (dy g) - x r^3 mean((dy g) x); one block per row
__global__ __launch_bounds__(256) void tr_rmsnorm_bwd_kernel(const float *x, const float *g, const float *r, const float *dy,
                                                             int d, float *dx)
{
    __shared__ float red[4];
    const int row = blockIdx.x;
    const float *xr = x + (size_t)row * d, *dyr = dy + (size_t)row * d;
    float s = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) s += dyr[i] * g[i] * xr[i];
    s = tr_block_sum(s, red) / (float)d;
    const float rr = r[row], r3 = rr * rr * rr;
    for (int i = threadIdx.x; i < d; i += 256) dx[(size_t)row * d + i] = rr * dyr[i] * g[i] - xr[i] * r3 * s;
}

// dg[j] (+)= sum_t dy[t][j] * x[t][j] * r[t]; a block of 1024 threads handles 64 columns, its 16 groups of
// 64 threads take every 16th row and their partial sums are added in group order
__global__ __launch_bounds__(1024) void tr_gain_grad_kernel(const float *x, const float *r, const float *dy, int T, int d, float *dg,
                                                            int accumulate)
{
    __shared__ float part[16][64];
    const int c = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + c;
    float s = 0.f;
    if (j < d)
        for (int t = grp; t < T; t += 16) s += dy[(size_t)t * d + j] * x[(size_t)t * d + j] * r[t];
    part[grp][c] = s;
    __syncthreads();
    if (grp == 0 && j < d) {
        float tot = 0.f;
#pragma unroll
        for (int g = 0; g < 16; g++) tot += part[g][c];
        dg[j] = accumulate ? dg[j] + tot : tot;
    }
}

// rotary embedding of the q and k parts of QKV [T][3d] at positions 0..T-1, pairs (i, i + hd/2);
// inverse rotates by minus the angle (the transpose of the rotation, for the backward pass)
__global__ void tr_rope_kernel(float *qkv, int T, int d, int hd, const float2 *tab, int inverse)
{
    const int half = hd >> 1;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per_row = (size_t)(d / hd) * half;
    if (i >= (size_t)T * per_row * 2) return;
    const int which = (int)(i / ((size_t)T * per_row));          // 0 = q, 1 = k
    const size_t j = i % ((size_t)T * per_row);
    const int t = (int)(j / per_row), rem = (int)(j % per_row), h = rem / half, p = rem % half;
    float2 cs = tab[(size_t)t * half + p];
    if (inverse) cs.y = -cs.y;
    float *v = qkv + (size_t)t * 3 * d + (size_t)which * d + (size_t)h * hd;
    const float a = v[p], b = v[p + half];
    v[p] = a * cs.x - b * cs.y;
    v[p + half] = b * cs.x + a * cs.y;
}

#define TR_T_MAX 2048   // longest training sequence: the attention row kernels keep a row of T weights in registers

// Attention over all positions at once goes through the contraction kernel, one product per head:
// S = Q.K^T, P = causal softmax(S / sqrt(hd)), O = P.V forward; dP = dO.V^T, dV = P^T.dO,
// dS = P (dP - rowsum(dP P)) / sqrt(hd), dQ = dS.K, dK = dS^T.Q backward.  The two kernels below are
// the row-wise pieces; both work in place on [H][T][T], one block per (row i, head h), and leave
// exact zeros above the diagonal.
__global__ __launch_bounds__(256) void tr_softmax_causal_kernel(float *P, int T, float scale)
{
    __shared__ float red[4];
    const int i = blockIdx.x, h = blockIdx.y, t = threadIdx.x;
    float *row = P + ((size_t)h * T + i) * T;
    float v[TR_T_MAX / 256];
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < TR_T_MAX / 256; c++) {
        const int j = t + 256 * c;
        v[c] = (j <= i) ? row[j] * scale : -INFINITY;      // j <= i < T
        mx = fmaxf(mx, v[c]);
    }
    mx = tr_block_max(mx, red);
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < TR_T_MAX / 256; c++) {
        v[c] = (t + 256 * c <= i) ? expf(v[c] - mx) : 0.f;
        sum += v[c];
    }
    sum = tr_block_sum(sum, red);
#pragma unroll
    for (int c = 0; c < TR_T_MAX / 256; c++) {
        const int j = t + 256 * c;
        if (j < T) row[j] = v[c] / sum;
    }
}

// dS[i][j] = P[i][j] * (dP[i][j] - sum_j dP[i][j] P[i][j]) * scale, in place on dP
__global__ __launch_bounds__(256) void tr_dsoftmax_kernel(const float *P, float *dP, int T, float scale)
{
    __shared__ float red[4];
    const int i = blockIdx.x, h = blockIdx.y, t = threadIdx.x;
    const float *prow = P + ((size_t)h * T + i) * T;
    float *drow = dP + ((size_t)h * T + i) * T;
    float p[TR_T_MAX / 256], g[TR_T_MAX / 256];
    float D = 0.f;
#pragma unroll
    for (int c = 0; c < TR_T_MAX / 256; c++) {
        const int j = t + 256 * c;
        p[c] = (j <= i) ? prow[j] : 0.f;
        g[c] = (j <= i) ? drow[j] : 0.f;
        D += p[c] * g[c];
    }
    D = tr_block_sum(D, red);
#pragma unroll
    for (int c = 0; c < TR_T_MAX / 256; c++) {
        const int j = t + 256 * c;
        if (j < T) drow[j] = p[c] * (g[c] - D) * scale;
    }
}

// Eq. 3 for one position: loss[t] = - sum_n p_n log q_n with p = softmax(zt[t]), q = softmax(z[t]);
// dz[t] = q - p (the gradient of the loss with respect to the draft logits).  One block per row.
__global__ __launch_bounds__(256) void tr_loss_kernel(const float *z, const float *zt, int V, float *dz, float *loss)
{
    __shared__ float red[4];
    const int row = blockIdx.x;
    const float *zr = z + (size_t)row * V, *tr = zt + (size_t)row * V;
    float mz = -INFINITY, mt = -INFINITY;
    for (int n = threadIdx.x; n < V; n += 256) { mz = fmaxf(mz, zr[n]); mt = fmaxf(mt, tr[n]); }
    mz = tr_block_max(mz, red);
    mt = tr_block_max(mt, red);
    float sz = 0.f, st = 0.f;
    for (int n = threadIdx.x; n < V; n += 256) { sz += expf(zr[n] - mz); st += expf(tr[n] - mt); }
    sz = tr_block_sum(sz, red);
    st = tr_block_sum(st, red);
    const float lz = logf(sz);
    float l = 0.f;
    for (int n = threadIdx.x; n < V; n += 256) {
        const float p = expf(tr[n] - mt) / st;
        const float lq = zr[n] - mz - lz;
        l -= p * lq;
        dz[(size_t)row * V + n] = expf(lq) - p;
    }
    l = tr_block_sum(l, red);
    if (threadIdx.x == 0) loss[row] = l;
}

// AdamW with bias correction and decoupled weight decay; c1 = 1 - beta1^step, c2 = 1 - beta2^step
__global__ void tr_adamw_kernel(float *w, const float *g, float *m, float *v, size_t n, float lr, float b1, float b2, float eps,
                                float wd, float c1, float c2)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float gi = g[i];
    const float mi = b1 * m[i] + (1.f - b1) * gi;
    const float vi = b2 * v[i] + (1.f - b2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    w[i] = w[i] * (1.f - lr * wd) - lr * (mi / c1) / (sqrtf(vi / c2) + eps);
}

// dst[i] = src[i] rounded to bfloat16 (nearest even), kept as fp32: what a bf16 checkpoint would hold
__global__ void tr_round_bf16_kernel(const float *src, int n, float *dst)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = bf2f(f2bf(src[i]));
}

// fp32 row-major [rows][K] <-> the arena's form of a matrix: bf16 MFMA tiles (the layout of
// pack_w_bf16_kernel) or fp32 rows, with source row r living at arena row map_row(r, row_off, mode)
// (mode 1 / 2: the interleaved gate / up rows of a feed-forward pair); K % 8 == 0 for tiles
__global__ void tr_unpack_bf16_kernel(const uint16_t *tiles, int rows, int K, int KS, int row_off, int mode, float *dst)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * K) return;
    const int r = (int)(i / K), k = (int)(i % K);
    dst[i] = bf2f(tiles[packed_u16_index(map_row(r, row_off, mode), k, KS)]);
}
// one thread per 16-byte unit of a tile: 8 consecutive columns of one row
__global__ void tr_pack_bf16_kernel(const float *src, int rows, int K, int KS, int row_off, int mode, uint16_t *tiles)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int K8 = K >> 3;
    if (i >= (size_t)rows * K8) return;
    const int r = (int)(i / K8), k = (int)(i % K8) * 8;
    const float4 a = *(const float4 *)(src + (size_t)r * K + k), b = *(const float4 *)(src + (size_t)r * K + k + 4);
    u32x4_t v;
    v[0] = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
    v[1] = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
    v[2] = (uint32_t)f2bf(b.x) | ((uint32_t)f2bf(b.y) << 16);
    v[3] = (uint32_t)f2bf(b.z) | ((uint32_t)f2bf(b.w) << 16);
    *(u32x4_t *)(tiles + packed_u16_index(map_row(r, row_off, mode), k, KS)) = v;
}
// the same for fp32 models; to_arena: master -> arena, else arena -> master
__global__ void tr_copy_rows_f32_kernel(float *master, float *arena, int rows, int K, int row_off, int mode, int to_arena)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * K) return;
    const int r = (int)(i / K), k = (int)(i % K);
    const size_t j = (size_t)map_row(r, row_off, mode) * K + k;
    if (to_arena) arena[j] = master[i]; else master[i] = arena[j];
}

// ---- element-wise pieces of the feed-forward and two-linear-map adapters --------------------
__device__ __forceinline__ float tr_sigmoid(float z) { return 1.f / (1.f + expf(-z)); }
// s = silu(u)
__global__ void tr_silu_kernel(const float *u, size_t n, float *s)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) s[i] = u[i] * tr_sigmoid(u[i]);
}
// du = ds * silu'(u), silu'(u) = sg (1 + u (1 - sg))
__global__ void tr_silu_bwd_kernel(const float *u, const float *ds, size_t n, float *du)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float z = u[i], sg = tr_sigmoid(z);
    du[i] = ds[i] * sg * (1.f + z * (1.f - sg));
}
// a = silu(g) * u
__global__ void tr_swiglu_kernel(const float *g, const float *u, size_t n, float *a)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) a[i] = g[i] * tr_sigmoid(g[i]) * u[i];
}
// dg = da * u * silu'(g), du = da * silu(g)
__global__ void tr_swiglu_bwd_kernel(const float *g, const float *u, const float *da, size_t n, float *dg, float *du)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float z = g[i], sg = tr_sigmoid(z), d = da[i];
    dg[i] = d * u[i] * sg * (1.f + z * (1.f - sg));
    du[i] = d * z * sg;
}
// a += b
__global__ void tr_add_kernel(float *a, const float *b, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) a[i] += b[i];
}
