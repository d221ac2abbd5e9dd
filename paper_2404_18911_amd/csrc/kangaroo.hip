// Host side of libkangaroo: the C ABI declared in include/kangaroo.h.  It owns no device memory;
// it carves the caller's arena / KV pool / scratch, launches the kernels of kernels.hip.h on the
// caller's stream, and runs the control flow of the draft-and-verify round (Section 3, Figure 2).
#include "kernels.hip.h"
#include "train.hip.h"

#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "kangaroo.h"

namespace {

constexpr size_t ALIGN = 256;
// Prompt rows handled per pass of the prompt kernels.  With the half-precision cache the projections
// run in workgroups of 128 rows x 8 TW weight tiles, one per compute unit at a time: a pass of 1024
// rows gives some launches 0.75 or 2.7 rounds of workgroups, a pass of 4096 rows 3 .. 11 rounds (a
// 4096-token prompt at the 7B shape: 122 ms in passes of 1024 rows, 109 in passes of 2048, 105 in one).
// The other cache types keep the 8-row-block kernels, whose attention needs page partials per block.
constexpr int PF_ROWS_MAX = 1024, PF_ROWS_MAX_HALF = 4096;
inline size_t up(size_t x, size_t a = ALIGN) { return (x + a - 1) / a * a; }

struct LayerW {
    size_t qkv, wo, gu, wd, g1, g2; // byte offsets into the arena
};

struct Phase { enum { NONE = 0, READY = 1, DRAFTING = 2, VERIFIED = 3, PLAIN = 4 }; };

// Workspace of the adapter's training step (byte offsets).  The parameter block, and likewise the
// gradient block and the two AdamW moment blocks, holds the adapter's tensors as fp32 in the order
// of train_tensors(): for the paper's adapter Wq, Wk, Wv (stacked, [3d][d]), Wo [d][d], g_in [d],
// g_last [d].
struct TrainLayout {
    size_t nparam = 0;
    size_t P = 0, G = 0, M = 0, V = 0;
    size_t F = 0, X = 0, Xn = 0, N = 0, QKV = 0, O = 0, H = 0, Mm = 0, Z = 0, Zt = 0, dZ = 0, rin = 0, rlast = 0, rfin = 0,
           Pm = 0, dS = 0, dMm = 0, dH = 0, dO = 0, dQKV = 0, dN = 0, loss = 0, part = 0,
           H1 = 0, Bn = 0, dB = 0, rpost = 0, Gt = 0, Ut = 0, Act = 0, dAct = 0, dGt = 0, dUt = 0;
    size_t part_floats = 0;
    size_t bytes = 0;
};

} // namespace

struct kg_ctx {
    kg_config c;
    bool bf;
    int esz;                 // bytes per stored weight element
    int kvt; int kvesz;      // KV cache element type (kg_config.kv_dtype) and its size
    int KSd, KSf;            // k-steps (32 features) of d_model and d_ffn
    int n_pages, logP;
    int n_cus = 256;         // compute units of the device (read at kg_bind)
    // arena layout
    std::vector<LayerW> lw;
    size_t a_qkv, a_wo, a_gin, a_glast, head, embed, gfinal, arena_bytes;
    // tensors of the other adapter architectures of Table 2 (allocated when adapter_kind has them)
    size_t a_head = 0, a_gpost = 0, a_gu = 0, a_wd = 0, a_w1 = 0, a_w2 = 0;
    int akind = 0;
    size_t kv_bytes, scratch_bytes;
    // scratch layout (byte offsets)
    size_t s_x0, s_x1, s_F, s_qkv, s_actX, s_actA, s_actF, s_ssq0, s_ssq1, s_opart, s_mxs, s_sms, s_cnt,
        s_dlog, s_tlog, s_tok, s_conf, s_pt, s_rope, s_invf, s_misc, s_hstat, s_dstat, s_tstat, s_acc;
    // prompt pass: device copy of the prompt and buffers for pf_rows rows at a time (bf16 weights)
    int pf_rows = 0;
    size_t s_ptok, s_px0, s_px1, s_pF, s_pqkv, s_pactX, s_pactA, s_pactF, s_pssq0, s_pssq1, s_popart, s_pmxs, s_psms,
        s_pcnt, s_pscale;
    // bindings
    char *arena = nullptr, *kv = nullptr, *scr = nullptr;
    hipStream_t stream = nullptr;
    hipEvent_t ev_fetch = nullptr;
    bool bound = false;
    std::vector<char> loaded; // per (kind, layer) flag
    std::vector<int> page_order;
    // pinned host staging
    int *h_tok = nullptr;
    float *h_conf = nullptr;
    // sequence state (see kg_get_state)
    int phase = Phase::NONE;
    int base = 0, adapter_len = 0, lag = 0, pending = -1;
    int n_drafts = 0, stopped = 0;
    int drafts[KG_MAX_ROWS];
    float confs[KG_MAX_ROWS];
    int targets[KG_MAX_ROWS];
    int n_target_rows = 0;
    int plain_len = 0;
    int spec_shallow = -1;   // index j of an early feature f_j already computed ahead of the host's decision
    // algorithmic bytes (weights streamed + cached keys / values read) by what the launches belong to:
    // 0 = self-draft model (shallow layers + adapter + head of a draft step), 1 = shallow-only pass
    // (the stopped token's next early feature), 2 = verification / plain forward, 3 = prompt pass
    double acct[4] = {0, 0, 0, 0};
    int acct_phase = 3;
    double spec_cost = 0;     // bytes of the run-ahead shallow pass still booked as shallow-only
    // adapter training (kg_train_*)
    char *tr = nullptr;
    TrainLayout tl;
    int tr_T = 0, tr_n = 0, tr_pending = 0;   // capacity, tokens of the last sequence, sequences in the gradient block
    long long tr_step = 0;
    // optional per-launch timing
    bool profiling = false;
    kg_profile prof;
    std::vector<hipEvent_t> ev_pool;
    struct Pending { int cls; double bytes; long long launches; size_t e0, e1; };
    std::vector<Pending> ev_pending;
    size_t ev_used = 0;
    char err[512];
};

namespace {

int fail(kg_ctx *ctx, int code, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define HIPCHK(ctx, call)                                                                            \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess) return fail(ctx, KG_EHIP, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)

#define KGCHK(call)                 \
    do {                            \
        int r_ = (call);            \
        if (r_ != KG_OK) return r_; \
    } while (0)

inline size_t act_bytes(int K) { return (size_t)((K + 31) / 32) * 1024; }
inline size_t packed_bytes(bool bf, int N, int K) { return bf ? (size_t)(N / 16) * ((K + 31) / 32) * 1024 : (size_t)N * K * 4; }

int ilog2(int v)
{
    int l = 0;
    while ((1 << l) < v) l++;
    return l;
}

void layout(kg_ctx *x)
{
    const kg_config &c = x->c;
    const int d = c.d_model, f = c.d_ffn, V = c.vocab, L = c.n_layers;
    size_t o = 0;
    auto take = [&](size_t b) { size_t r = o; o += up(b); return r; };
    x->lw.resize(L);
    for (int i = 0; i < L; i++) {
        x->lw[i].qkv = take(packed_bytes(x->bf, 3 * d, d));
        x->lw[i].wo = take(packed_bytes(x->bf, d, d));
        x->lw[i].gu = take(packed_bytes(x->bf, 2 * f, d));
        x->lw[i].wd = take(packed_bytes(x->bf, d, f));
        x->lw[i].g1 = take((size_t)d * 4);
        x->lw[i].g2 = take((size_t)d * 4);
    }
    x->a_qkv = x->a_wo = 0;
    if (x->akind != KG_ADAPTER_MLP) {
        x->a_qkv = take(packed_bytes(x->bf, 3 * d, d));
        x->a_wo = take(packed_bytes(x->bf, d, d));
    } else {
        x->a_w1 = take(packed_bytes(x->bf, d, d));
        x->a_w2 = take(packed_bytes(x->bf, d, d));
    }
    if (x->akind == KG_ADAPTER_LAYER) {
        x->a_gu = take(packed_bytes(x->bf, 2 * f, d));
        x->a_wd = take(packed_bytes(x->bf, d, f));
        x->a_gpost = take((size_t)d * 4);
    }
    if (x->akind == KG_ADAPTER_ATTN_HEAD || x->akind == KG_ADAPTER_MLP) x->a_head = take(packed_bytes(x->bf, V, d));
    x->a_gin = take((size_t)d * 4);
    x->a_glast = take((size_t)d * 4);
    x->head = take(packed_bytes(x->bf, V, d));
    x->embed = take((size_t)V * d * x->esz);
    x->gfinal = take((size_t)d * 4);
    x->arena_bytes = o;

    x->kv_bytes = up((size_t)x->n_pages * (L + 1) * c.n_heads * 2 * c.kv_page_tokens * c.head_dim * x->kvesz);

    o = 0;
    x->s_x0 = take((size_t)KG_ROWS * d * 4);
    x->s_x1 = take((size_t)KG_ROWS * d * 4);
    x->s_F = take((size_t)(KG_ROWS + 1) * d * 4); // row 0: lagged feature, rows 1..8: f_0..f_7
    x->s_qkv = take((size_t)KG_ROWS * 3 * d * 4);
    x->s_actX = take(act_bytes(d));
    x->s_actA = take(act_bytes(d));
    x->s_actF = take(act_bytes(f));
    x->s_ssq0 = take((size_t)(d / 16) * KG_ROWS * 4);
    x->s_ssq1 = take((size_t)(d / 16) * KG_ROWS * 4);
    x->s_opart = take((size_t)c.n_heads * x->n_pages * KG_ROWS * c.head_dim * 4);
    x->s_mxs = take((size_t)c.n_heads * x->n_pages * KG_ROWS * 4);
    x->s_sms = take((size_t)c.n_heads * x->n_pages * KG_ROWS * 4);
    x->s_cnt = take((size_t)c.n_heads * 4);
    x->s_dlog = take((size_t)KG_ROWS * V * 4);
    x->s_tlog = take((size_t)KG_ROWS * V * 4);
    x->s_tok = take(KG_ROWS * 8);            // tokens, then confidences: one 64-byte block, one copy to the host
    x->s_conf = x->s_tok + KG_ROWS * 4;
    x->s_pt = take((size_t)x->n_pages * 4);
    x->s_rope = take((size_t)c.max_seq * (c.head_dim / 2) * 8);
    x->s_invf = take((size_t)(c.head_dim / 2) * 8);
    x->s_misc = take((size_t)2 * d * 4);
    x->s_hstat = take((size_t)(V / 16) * KG_ROWS * 4 * 4);
    x->s_dstat = take(KG_ROWS * 2 * 4);
    x->s_tstat = take(KG_ROWS * 2 * 4);
    x->s_acc = take(2 * 4);
    x->s_ptok = take((size_t)c.max_seq * 4);
    x->pf_rows = 0;
    if (x->bf) {
        const bool half = x->kvt == 2;          // prompt attention on the matrix units: no page partials
        x->pf_rows = std::min(half ? PF_ROWS_MAX_HALF : PF_ROWS_MAX, (c.max_seq + KG_ROWS - 1) / KG_ROWS * KG_ROWS);
        const size_t R = x->pf_rows, nb = R / KG_ROWS, nbp = half ? 1 : nb;
        x->s_px0 = take(R * d * 4);
        x->s_px1 = take(R * d * 4);
        x->s_pF = take(R * d * 4);
        x->s_pqkv = take(R * 3 * d * 4);
        x->s_pactX = take(nb * act_bytes(d));
        x->s_pactA = take(nb * act_bytes(d));
        x->s_pactF = take(nb * act_bytes(f));
        x->s_pssq0 = take(nb * (d / 16) * KG_ROWS * 4);
        x->s_pssq1 = take(nb * (d / 16) * KG_ROWS * 4);
        x->s_popart = take(nbp * c.n_heads * x->n_pages * KG_ROWS * c.head_dim * 4);
        x->s_pmxs = take(nbp * c.n_heads * x->n_pages * KG_ROWS * 4);
        x->s_psms = take(nbp * c.n_heads * x->n_pages * KG_ROWS * 4);
        x->s_pcnt = take(nb * c.n_heads * 4);
        x->s_pscale = take(R * 4);
    }
    x->scratch_bytes = o;
}

template <typename T> inline T *at(char *basep, size_t off) { return reinterpret_cast<T *>(basep + off); }

int check_launch(kg_ctx *x, const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(x, KG_EHIP, "launch %s: %s", what, hipGetErrorString(e));
    return KG_OK;
}

// ---- optional per-launch timing -----------------------------------------------------------------

size_t prof_event(kg_ctx *x)
{
    if (x->ev_used == x->ev_pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return (size_t)-1;
        x->ev_pool.push_back(e);
    }
    return x->ev_used++;
}

// A run of consecutive launches of one class shares one pair of events: the pair costs about as
// much device time as a small kernel, so bracketing every launch would inflate what it measures.
// The run is closed by the first launch of another class, or by prof_flush before the host waits.
void prof_flush(kg_ctx *x)
{
    if (!x->profiling || x->ev_pending.empty()) return;
    auto &p = x->ev_pending.back();
    if (p.e1 != (size_t)-1) return;
    size_t e1 = prof_event(x);
    if (e1 == (size_t)-1) { x->ev_pending.pop_back(); return; }
    (void)hipEventRecord(x->ev_pool[e1], x->stream);
    x->ev_pending.back().e1 = e1;
}

struct ProfScope {
    ProfScope(kg_ctx *x, int cls, double bytes)
    {
        if (!x->profiling) return;
        if (!x->ev_pending.empty() && x->ev_pending.back().e1 == (size_t)-1 && x->ev_pending.back().cls == cls) {
            x->ev_pending.back().bytes += bytes;
            x->ev_pending.back().launches++;
            return;
        }
        prof_flush(x);
        size_t e0 = prof_event(x);
        if (e0 == (size_t)-1) return;
        (void)hipEventRecord(x->ev_pool[e0], x->stream);
        x->ev_pending.push_back({cls, bytes, 1, e0, (size_t)-1});
    }
};

void prof_collect(kg_ctx *x)   // call after prof_flush and a synchronisation of the stream
{
    for (auto &p : x->ev_pending) {
        float ms = 0.f;
        if (p.e1 != (size_t)-1 && hipEventElapsedTime(&ms, x->ev_pool[p.e0], x->ev_pool[p.e1]) == hipSuccess) {
            x->prof.launches[p.cls] += p.launches;
            x->prof.seconds[p.cls] += ms * 1e-3;
            x->prof.bytes[p.cls] += p.bytes;
        }
    }
    x->ev_pending.clear();
    x->ev_used = 0;
}

// ---- kernel launch helpers ---------------------------------------------------------------------

int launch_gemv(kg_ctx *x, size_t w_off, int N, int K, const void *act, const Epi &e)
{
    if (N % 16) return fail(x, KG_EINVAL, "projection rows %d not a multiple of 16", N);
    ProfScope ps(x, 0, (double)N * K * x->esz);
    x->acct[x->acct_phase] += (double)N * K * x->esz;
    if (x->bf)
        hipLaunchKernelGGL(gemv_bf16_kernel, dim3(N / 16), dim3(64 * GEMV_WAVES), 0, x->stream,
                           at<const u32x4_t>(x->arena, w_off), (K + 31) / 32, e.M, (const u32x4_t *)act, e.ssq_in, e.nt_in,
                           e.N, e.kind == EPI_RESID ? e.res : nullptr, e.gain, e);
    else
        hipLaunchKernelGGL(gemv_f32_kernel, dim3(N / 16), dim3(256), 0, x->stream, at<const float>(x->arena, w_off),
                           K, (const float *)act, e);
    return check_launch(x, "gemv");
}

int launch_pack_rows(kg_ctx *x, const int *tokens, const float *rows, int M, const float *gain, float *xout,
                     void *act, float *ssq, const int *tok_dev = nullptr)
{
    Tok8 tk;
    for (int i = 0; i < KG_ROWS; i++) tk.t[i] = (tokens && i < M) ? tokens[i] : 0;
    tk.vocab = x->c.vocab;
    const void *emb = (tokens || tok_dev) ? (const void *)(x->arena + x->embed) : nullptr;
    const int d = x->c.d_model;
    ProfScope ps(x, 2, 0.0);
    if (x->bf)
        hipLaunchKernelGGL(pack_rows_kernel<true>, dim3(d / 16), dim3(128), 0, x->stream, emb, tk, tok_dev, rows, d, M,
                           gain, xout, act, ssq);
    else
        hipLaunchKernelGGL(pack_rows_kernel<false>, dim3(d / 16), dim3(128), 0, x->stream, emb, tk, tok_dev, rows, d, M,
                           gain, xout, act, ssq);
    return check_launch(x, "pack_rows");
}

template <typename T, int HD, bool BF>
void launch_attn_rows(const AttnArgs &a, dim3 grid, int rows, hipStream_t stream)
{
    // rows = row capacity of the instantiation (1, 2, 4 or 8 >= rows of a block)
    if (rows <= 1) hipLaunchKernelGGL((attn_kernel<T, HD, BF, 1>), grid, dim3(512), 0, stream, a);
    else if (rows <= 2) hipLaunchKernelGGL((attn_kernel<T, HD, BF, 2>), grid, dim3(512), 0, stream, a);
    else if (rows <= 4) hipLaunchKernelGGL((attn_kernel<T, HD, BF, 4>), grid, dim3(512), 0, stream, a);
    else hipLaunchKernelGGL((attn_kernel<T, HD, BF, 8>), grid, dim3(512), 0, stream, a);
}

int launch_attn_args(kg_ctx *x, const AttnArgs &a, dim3 grid, int rows)
{
    const int hd = x->c.head_dim;
    if (x->bf && x->kvt == 2) {
        if (hd == 128) launch_attn_rows<kvhalf_t, 128, true>(a, grid, rows, x->stream);
        else launch_attn_rows<kvhalf_t, 64, true>(a, grid, rows, x->stream);
    } else if (x->bf && x->kvt == 1) {
        if (hd == 128) launch_attn_rows<uint16_t, 128, true>(a, grid, rows, x->stream);
        else launch_attn_rows<uint16_t, 64, true>(a, grid, rows, x->stream);
    } else if (x->bf) {
        if (hd == 128) launch_attn_rows<float, 128, true>(a, grid, rows, x->stream);
        else launch_attn_rows<float, 64, true>(a, grid, rows, x->stream);
    } else {
        if (hd == 128) launch_attn_rows<float, 128, false>(a, grid, rows, x->stream);
        else launch_attn_rows<float, 64, false>(a, grid, rows, x->stream);
    }
    return check_launch(x, "attention");
}

AttnArgs attn_args(kg_ctx *x, int slot, int pos0, int M)
{
    const kg_config &c = x->c;
    AttnArgs a;
    memset(&a, 0, sizeof(a));
    a.qkv = at<const float>(x->scr, x->s_qkv);
    a.d = c.d_model; a.H = c.n_heads; a.M = M; a.pos0 = pos0; a.P = c.kv_page_tokens; a.logP = x->logP;
    a.page_table = at<const int>(x->scr, x->s_pt);
    for (int i = 0; i < 16; i++) a.pages[i] = i < x->n_pages ? x->page_order[i] : 0;
    a.kv = x->kv; a.slot = slot; a.n_slots = c.n_layers + 1;
    a.rope = at<const float2>(x->scr, x->s_rope);
    a.opart = at<float>(x->scr, x->s_opart); a.mxs = at<float>(x->scr, x->s_mxs); a.sms = at<float>(x->scr, x->s_sms);
    a.cnt = at<int>(x->scr, x->s_cnt);
    a.S = (pos0 + M + c.kv_page_tokens - 1) >> x->logP;
    a.act_out = x->scr + x->s_actA;
    return a;
}

int launch_attn(kg_ctx *x, int slot, int pos0, int M, int append_only)
{
    const kg_config &c = x->c;
    AttnArgs a = attn_args(x, slot, pos0, M);
    a.append_only = append_only;
    const double kv_read = append_only ? 0.0 : (double)(pos0 + M) * 2 * c.d_model * x->kvesz;
    ProfScope ps(x, 1, kv_read);
    x->acct[x->acct_phase] += kv_read;
    return launch_attn_args(x, a, dim3(c.n_heads, a.S), M);
}

Epi epi_base(kg_ctx *x, int kind, int M, int N);

// ---- prompt pass (dense MFMA projections over many 8-row blocks) ---------------------------------

enum { PF_PLAN_TW1_RB8 = 17 };     // pf_gemm_plan: TW 1 with workgroups of 64 rows
int pf_gemm_plan(const kg_ctx *x, int N, int K, int T);

int launch_pf_pack(kg_ctx *x, const int *tok_dev, const float *rows, int T, const float *gain, float *xout)
{
    const int d = x->c.d_model, nb = (T + KG_ROWS - 1) / KG_ROWS;
    Tok8 tk;
    memset(&tk, 0, sizeof(tk));
    tk.vocab = x->c.vocab;
    const void *emb = tok_dev ? (const void *)(x->arena + x->embed) : nullptr;
    ProfScope ps(x, 2, 0.0);
    // the rows feed a q,k,v projection: stored in the layout its kernel reads
    hipLaunchKernelGGL(pack_rows_kernel<true>, dim3(d / 16, nb), dim3(128), 0, x->stream, emb, tk, tok_dev, rows, d, T, gain,
                       xout, (void *)(x->scr + x->s_pactX), at<float>(x->scr, x->s_pssq0), act_bytes(d),
                       (d / 16) * KG_ROWS, pf_gemm_plan(x, 3 * d, d, T) ? 1 : 0);
    return check_launch(x, "prompt pack_rows");
}

// Y[T][N] = X[T][K] . W^T with the epilogue e applied per 8-row block; in/out block strides follow
// the prompt buffers (activation tiles of K features per block, d/16 tile sums per block)
// Which kernel multiplies a prompt pass of T rows by a matrix [N][K]: 0 = the 8-row-block kernels
// (gemm_prefill_body: rows bit-identical to one-token decoding), else the TW of gemm_prefill2_body.
// The answer also fixes the layout in which the producer of the projection's input has to store it
// (pf_act_ptr: the pair layout for gemm_prefill2_body).
int pf_gemm_plan(const kg_ctx *x, int N, int K, int T)
{
    // long passes with the half-precision cache only (its prompt rows are not bit-identical to decoded rows anyway)
    if (T < 256 || x->kvt != 2 || (K + 31) / 32 > PF2_KS_MAX) return 0;
    // Workgroups of 8 * TW weight tiles x 128 rows.  TW is the one with the least operand traffic: per
    // k-step every row group fetches all NT weight tiles and every workgroup its 16 activation tiles,
    // and a last round of workgroups that fills only part of the device costs a whole round; beside the
    // traffic, the kernels that read the next k-step's operands under the current one's multiplications
    // (TW 1 and 2) take 0.95 and 1.0 of the model's time and TW 4 takes 1.2.  Measured at the 7B shape under a
    // kernel trace, microseconds per launch for TW 1 / 2 / 4: 1024 rows: q,k,v 190 / 191 / 180, gate+up 359 / 296 /
    // 364, o_proj and down_proj 119 / 164 / 313; 2048 rows: q,k,v 390 / 323 / 367, gate+up 686 / 599 / 589, o_proj
    // and down_proj 245 / 204 / 331 (the model picks the fastest of each); 256 rows: q,k,v TW 1 58, gate+up TW 2 91.
    // At 4096 rows the model picks TW 4 for every projection (3 .. 11 full rounds of workgroups): a 4096-token
    // prompt took 104.5 ms so, 108.4 ms with TW 2 for gate+up and 114.2 ms with TW 2 for q,k,v as well.
    const int NT = N / 16, nb = (T + KG_ROWS - 1) / KG_ROWS, gx2 = (nb + 15) / 16;
    int best_tw = 1;
    double best_cost = -1.0, best_wgs = 0.0;
    for (int tw = 4; tw >= 1; tw >>= 1) {
        const int gy = (NT + 8 * tw - 1) / (8 * tw);
        const double wgs = (double)gx2 * gy;
        const double rounds = std::ceil(wgs / x->n_cus);
        const double cost = ((double)NT * gx2 + 16.0 * wgs) * rounds * x->n_cus / wgs * (tw == 4 ? 1.2 : tw == 2 ? 1.0 : 0.95);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_tw = tw; best_wgs = wgs; }
    }
    // few weight tiles (o_proj and down_proj at 256 rows: 64 workgroups of 128 rows): workgroups of 64 rows
    // where those reach that fill (70 us per launch against 84 us of the 8-row-block kernel), else that kernel.
    // A workgroup of 64 rows takes 0.55 of the time of one of 128 rows, so the 64-row kernel also wins where it
    // needs no more rounds of workgroups than TW 1 does (o_proj and down_proj at 512 rows: 256 workgroups instead
    // of 128, a 512-token prompt 15.9 -> 14.6 ms; at 768 rows 384 instead of 192: two rounds, no gain).
    const double wgs8 = (double)((nb + 7) / 8) * ((NT + 7) / 8);
    if (best_wgs >= 0.45 * x->n_cus) {
        if (best_tw == 1 && 0.55 * std::ceil(wgs8 / x->n_cus) < std::ceil(best_wgs / x->n_cus)) return PF_PLAN_TW1_RB8;
        return best_tw;
    }
    return wgs8 >= 0.45 * x->n_cus ? PF_PLAN_TW1_RB8 : 0;
}

int launch_pf_gemm(kg_ctx *x, size_t w_off, int N, int K, const void *act, int T, const Epi &e, bool ssq_in, bool ssq_out,
                   int act_out_K)
{
    if (N % 16) return fail(x, KG_EINVAL, "projection rows %d not a multiple of 16", N);
    PfArgs a;
    memset(&a, 0, sizeof(a));
    a.W = at<const u32x4_t>(x->arena, w_off);
    a.KS = (K + 31) / 32; a.NT = N / 16;
    a.act = (const u32x4_t *)act; a.act_blk = act_bytes(K) / 16; a.T = T;
    const int sq = (x->c.d_model / 16) * KG_ROWS;
    a.ssq_in_blk = ssq_in ? sq : 0; a.ssq_out_blk = ssq_out ? sq : 0;
    a.act_out_blk = act_out_K ? act_bytes(act_out_K) : 0;
    const int nb = (T + KG_ROWS - 1) / KG_ROWS;
    if (const int plan = pf_gemm_plan(x, N, K, T)) {
        const int best_tw = plan == PF_PLAN_TW1_RB8 ? 1 : plan;
        a.gx = plan == PF_PLAN_TW1_RB8 ? (nb + 7) / 8 : (nb + 15) / 16;
        a.gy = (a.NT + 8 * best_tw - 1) / (8 * best_tw);
        const int groups = a.gx * 8 * ((a.gy + 7) / 8);
        Epi e2 = e;
        if (ssq_in) {       // the rows' RMS scales once per pass, not once per workgroup
            float *scale = at<float>(x->scr, x->s_pscale);
            hipLaunchKernelGGL(pf_rms_scale_kernel, dim3(nb), dim3(512), 0, x->stream, e.ssq_in, a.ssq_in_blk, e.nt_in, T, e.inv_d,
                               e.eps, scale);
            KGCHK(check_launch(x, "prompt row scales"));
            e2.scale_in = scale;
        }
        ProfScope ps(x, 3, 2.0 * T * (double)N * K);
        if (plan == PF_PLAN_TW1_RB8) hipLaunchKernelGGL(gemm_prefill2_kernel_tw1_rb8, dim3(groups), dim3(768), 0, x->stream, a, e2);
        else if (best_tw == 4) hipLaunchKernelGGL(gemm_prefill2_kernel_tw4, dim3(groups), dim3(768), 0, x->stream, a, e2);
        else if (best_tw == 2) hipLaunchKernelGGL(gemm_prefill2_kernel_tw2, dim3(groups), dim3(768), 0, x->stream, a, e2);
        else hipLaunchKernelGGL(gemm_prefill2_kernel_tw1, dim3(groups), dim3(768), 0, x->stream, a, e2);
        return check_launch(x, "prompt projection");
    }
    // two weight tiles per multiplying wave where that still leaves enough workgroups for the device
    const int tw = a.NT >= 512 ? 2 : 1;
    a.gy = (a.NT + 8 * tw - 1) / (8 * tw);
    // row groups of 8 blocks; of 4 where 8 would give fewer workgroups than the device has compute units
    int cbw = PF_CBW;
    if (tw == 1 && ((nb + PF_CBW - 1) / PF_CBW) * a.gy < x->n_cus && nb > 4) cbw = 4;
    a.gx = (nb + cbw - 1) / cbw;
    const int groups = a.gx * 8 * ((a.gy + 7) / 8);
    ProfScope ps(x, 3, 2.0 * T * (double)N * K);
    if (tw == 2) hipLaunchKernelGGL(gemm_prefill_kernel_tw2, dim3(groups), dim3(768), 0, x->stream, a, e);
    else if (cbw == 4) hipLaunchKernelGGL(gemm_prefill_kernel_tw1_cb4, dim3(groups), dim3(768), 0, x->stream, a, e);
    else hipLaunchKernelGGL(gemm_prefill_kernel_tw1, dim3(groups), dim3(768), 0, x->stream, a, e);
    return check_launch(x, "prompt projection");
}

// One decoder block (or the adapter's key/value projection when kv_only) on T prompt rows at pos0.
// In: pactX = x_in * g_attn, pssq0 = tile sums of x_in.  Out: x rows in x_out, pactX = x_out *
// next_gain, pssq0 = tile sums of x_out.  Every row's arithmetic is that of the one-token kernels.
int pf_block(kg_ctx *x, int slot, size_t qkv_off, size_t wo_off, size_t gu_off, size_t wd_off, const float *g2, int T,
             int pos0, const float *x_in, float *x_out, const float *next_gain, bool kv_only)
{
    const kg_config &c = x->c;
    const int d = c.d_model, f = c.d_ffn, nb = (T + KG_ROWS - 1) / KG_ROWS;
    float *ssq0 = at<float>(x->scr, x->s_pssq0), *ssq1 = at<float>(x->scr, x->s_pssq1);
    void *actX = x->scr + x->s_pactX, *actA = x->scr + x->s_pactA, *actF = x->scr + x->s_pactF;
    float *x_mid = at<float>(x->scr, x->s_px1);

    Epi e = epi_base(x, EPI_PLAIN, KG_ROWS, 3 * d);
    e.ssq_in = ssq0; e.out = at<float>(x->scr, x->s_pqkv);
    KGCHK(launch_pf_gemm(x, qkv_off, 3 * d, d, actX, T, e, true, false, 0));

    // all rows' keys and values go to the cache first; then every 8-row block attends to the cache
    AttnArgs a = attn_args(x, slot, pos0, T);
    a.qkv = at<const float>(x->scr, x->s_pqkv);
    a.opart = at<float>(x->scr, x->s_popart); a.mxs = at<float>(x->scr, x->s_pmxs); a.sms = at<float>(x->scr, x->s_psms);
    a.cnt = at<int>(x->scr, x->s_pcnt);
    a.act_out = actA; a.act_blk_bytes = act_bytes(d);
    a.append_only = 1; a.append_all = 1;
    {
        ProfScope ps(x, 1, 0.0);
        KGCHK(launch_attn_args(x, a, dim3(c.n_heads, 1, nb), KG_ROWS));
    }
    if (kv_only) return KG_OK;
    if (x->kvt == 2) {
        // half-precision cache: the prompt rows' attention runs on the matrix units
        PfAttnArgs pa;
        memset(&pa, 0, sizeof(pa));
        pa.qkv = at<const float>(x->scr, x->s_pqkv);
        pa.d = d; pa.H = c.n_heads; pa.T = T; pa.pos0 = pos0; pa.logP = x->logP;
        pa.page_table = at<const int>(x->scr, x->s_pt);
        pa.kv = (const kvhalf_t *)x->kv; pa.slot = slot; pa.n_slots = c.n_layers + 1;
        pa.rope = at<const float2>(x->scr, x->s_rope);
        pa.act_out = actA; pa.act_blk_bytes = act_bytes(d);
        pa.act_pair = pf_gemm_plan(x, d, d, T) ? 1 : 0;               // read by the output projection
        ProfScope ps(x, 1, 0.0);
        // workgroups of 128 rows (8 waves, a compute unit each) where those alone fill the device, else of 64 rows
        if ((size_t)c.n_heads * ((T + 127) / 128) >= (size_t)x->n_cus) {
            const dim3 grid(c.n_heads, (T + 127) / 128);
            if (c.head_dim == 128) hipLaunchKernelGGL((pf_attn_kernel<128, 8>), grid, dim3(512), 0, x->stream, pa);
            else hipLaunchKernelGGL((pf_attn_kernel<64, 8>), grid, dim3(512), 0, x->stream, pa);
        } else {
            const dim3 grid(c.n_heads, (T + 63) / 64);
            if (c.head_dim == 128) hipLaunchKernelGGL((pf_attn_kernel<128, 4>), grid, dim3(256), 0, x->stream, pa);
            else hipLaunchKernelGGL((pf_attn_kernel<64, 4>), grid, dim3(256), 0, x->stream, pa);
        }
        KGCHK(check_launch(x, "prompt attention"));
    } else {
        a.append_only = 0; a.append_all = 0; a.preappended = 1;
        ProfScope ps(x, 1, 0.0);
        KGCHK(launch_attn_args(x, a, dim3(c.n_heads, a.S, nb), KG_ROWS));
    }

    e = epi_base(x, EPI_RESID, KG_ROWS, d);
    e.res = x_in; e.xout = x_mid; e.act_out = actX; e.act_K = d; e.gain = g2; e.ssq_out = ssq1;
    e.act_pair = pf_gemm_plan(x, 2 * f, d, T) ? 1 : 0;                // read by gate+up
    KGCHK(launch_pf_gemm(x, wo_off, d, d, actA, T, e, false, true, d));

    e = epi_base(x, EPI_SWIGLU, KG_ROWS, 2 * f);
    e.ssq_in = ssq1; e.act_out = actF; e.act_K = f;
    e.act_pair = pf_gemm_plan(x, d, f, T) ? 1 : 0;                    // read by down_proj
    KGCHK(launch_pf_gemm(x, gu_off, 2 * f, d, actX, T, e, true, false, f));

    e = epi_base(x, EPI_RESID, KG_ROWS, d);
    e.res = x_mid; e.xout = x_out; e.act_out = next_gain ? actX : nullptr; e.act_K = d; e.gain = next_gain;
    e.ssq_out = ssq0;
    e.act_pair = pf_gemm_plan(x, 3 * d, d, T) ? 1 : 0;                // read by the next block's q,k,v
    KGCHK(launch_pf_gemm(x, wd_off, d, f, actF, T, e, false, true, next_gain ? d : 0));
    return KG_OK;
}

// Full model M^b and the adapter's cache on prompt rows pos0..pos0+T-1 (token ids in the device
// copy of the prompt).  Returns the device rows holding the last layer's output.
int pf_rows_pass(kg_ctx *x, int pos0, int T, const float **x_last)
{
    const kg_config &c = x->c;
    const int L = c.n_layers, l = c.exit_layer;
    float *x0 = at<float>(x->scr, x->s_px0), *F = at<float>(x->scr, x->s_pF);
    KGCHK(launch_pf_pack(x, at<const int>(x->scr, x->s_ptok) + pos0, nullptr, T, at<const float>(x->arena, x->lw[0].g1), x0));
    const float *xin = x0;
    for (int i = 0; i < L; i++) {
        const LayerW &w = x->lw[i];
        float *xout = (i == l - 1) ? F : x0;           // early features of all rows (Section 3.1)
        const float *ng = (i == L - 1) ? nullptr : at<const float>(x->arena, x->lw[i + 1].g1);
        KGCHK(pf_block(x, i, w.qkv, w.wo, w.gu, w.wd, at<const float>(x->arena, w.g2), T, pos0, xin, xout, ng, false));
        xin = xout;
    }
    *x_last = xin;
    // adapter: keys and values of every prompt position (its attention output is not needed here);
    // the adapter made of two linear maps keeps no cache
    if (x->akind == KG_ADAPTER_MLP) return KG_OK;
    KGCHK(launch_pf_pack(x, nullptr, F, T, at<const float>(x->arena, x->a_gin), nullptr));
    return pf_block(x, L, x->a_qkv, 0, 0, 0, nullptr, T, pos0, nullptr, nullptr, nullptr, true);
}

Epi epi_base(kg_ctx *x, int kind, int M, int N)
{
    Epi e;
    memset(&e, 0, sizeof(e));
    e.kind = kind; e.M = M; e.N = N;
    e.inv_d = 1.f / (float)x->c.d_model;
    e.eps = x->c.rms_eps;
    e.nt_in = x->c.d_model / 16;
    return e;
}

// Attention sub-layer + (optionally) feed-forward sub-layer of one block on M rows at pos0.
// In:  actX = x_in * g_attn (packed), ssq0 = tile sums of squares of x_in, x_in fp32 rows.
// Out: x rows in x_out; actX = x_out * next_gain if next_gain, ssq0 = tile sums of x_out.
int run_block(kg_ctx *x, int slot, size_t qkv_off, size_t wo_off, size_t gu_off, size_t wd_off, const float *g2,
              int M, int pos0, const float *x_in, float *x_out, const float *next_gain, bool with_ffn)
{
    const kg_config &c = x->c;
    const int d = c.d_model, f = c.d_ffn;
    float *ssq0 = at<float>(x->scr, x->s_ssq0), *ssq1 = at<float>(x->scr, x->s_ssq1);
    void *actX = x->scr + x->s_actX, *actA = x->scr + x->s_actA, *actF = x->scr + x->s_actF;
    float *x_mid = with_ffn ? at<float>(x->scr, x->s_x1) : x_out;

    Epi e = epi_base(x, EPI_PLAIN, M, 3 * d);
    e.ssq_in = ssq0; e.out = at<float>(x->scr, x->s_qkv);
    KGCHK(launch_gemv(x, qkv_off, 3 * d, d, actX, e));
    KGCHK(launch_attn(x, slot, pos0, M, 0));

    e = epi_base(x, EPI_RESID, M, d);
    e.res = x_in; e.xout = x_mid; e.act_out = actX; e.act_K = d;
    if (with_ffn) { e.gain = g2; e.ssq_out = ssq1; }
    else { e.gain = next_gain; e.ssq_out = ssq0; if (!next_gain) e.act_out = nullptr; }
    KGCHK(launch_gemv(x, wo_off, d, d, actA, e));
    if (!with_ffn) return KG_OK;

    e = epi_base(x, EPI_SWIGLU, M, 2 * f);
    e.ssq_in = ssq1; e.act_out = actF; e.act_K = f;
    KGCHK(launch_gemv(x, gu_off, 2 * f, d, actX, e));

    e = epi_base(x, EPI_RESID, M, d);
    e.res = x_mid; e.xout = x_out; e.act_out = next_gain ? actX : nullptr; e.act_K = d; e.gain = next_gain;
    e.ssq_out = ssq0;
    KGCHK(launch_gemv(x, wd_off, d, f, actF, e));
    return KG_OK;
}

// Decoder blocks lo..hi-1.  x_first: fp32 rows feeding block lo (already packed into actX/ssq0
// with norm1[lo]); the result rows land in x_last; final_gain prepares actX for what follows.
int run_layers(kg_ctx *x, int lo, int hi, int M, int pos0, const float *x_first, float *x_last,
               const float *final_gain)
{
    float *x0 = at<float>(x->scr, x->s_x0);
    const float *xin = x_first;
    for (int i = lo; i < hi; i++) {
        const LayerW &w = x->lw[i];
        bool last = (i == hi - 1);
        float *xout = last ? x_last : x0;
        const float *ng = last ? final_gain : at<const float>(x->arena, x->lw[i + 1].g1);
        KGCHK(run_block(x, i, w.qkv, w.wo, w.gu, w.wd, at<const float>(x->arena, w.g2), M, pos0, xin, xout, ng, true));
        xin = xout;
    }
    return KG_OK;
}

// LM head on the rows packed in actX (+ssq0): logits rows (m + row_shift) of `logits`, then
// arg-max and top-1 probability of rows 0..n_out-1 into the device tok/conf arrays.
// u: per-row uniform numbers for sampling (mode 1), stat: where the rows' (max, sum exp) go.
int run_head(kg_ctx *x, int M, int row_shift, float *logits, int n_out, float inv_temp, int mode = 0,
             const USrc *us = nullptr, int purpose = 0, float *stat = nullptr, bool draft = false)
{
    // the draft head is the adapter's own where its architecture has one (Table 2), else the shared LM head
    const size_t head_off = (draft && x->a_head) ? x->a_head : x->head;
    Epi e = epi_base(x, EPI_HEAD, M, x->c.vocab);
    e.ssq_in = at<float>(x->scr, x->s_ssq0); e.out = logits; e.row_shift = row_shift;
    e.hstat = at<float>(x->scr, x->s_hstat); e.inv_temp = inv_temp;
    KGCHK(launch_gemv(x, head_off, x->c.vocab, x->c.d_model, x->scr + x->s_actX, e));
    ProfScope ps(x, 2, 0.0);
    USrc uu;
    if (us) uu = *us; else memset(&uu, 0, sizeof(uu));
    hipLaunchKernelGGL(head_final_kernel, dim3(n_out), dim3(1024), 0, x->stream, at<const float>(x->scr, x->s_hstat),
                       x->c.vocab / 16, (const float *)logits, x->c.vocab, inv_temp, mode, uu, purpose, at<int>(x->scr, x->s_tok),
                       at<float>(x->scr, x->s_conf), stat ? stat : at<float>(x->scr, x->s_tstat));
    return check_launch(x, "head_final");
}

// Sampling mode: row `row` of a launch decides the token at absolute position pos.  With a table
// of uniform numbers from the caller its entries for up to two purposes are copied into the launch's
// arguments; otherwise the kernels evaluate the generator at (seed; position, purpose) themselves.
int usrc_row(kg_ctx *x, const kg_params *p, USrc &us, int row, int pos, int purpose0, int purpose1 = -1)
{
    us.pos[row] = pos;
    if (p->mode != 1) return KG_OK;
    us.from_seed = p->uniforms ? 0 : 1;
    us.k0 = (uint32_t)p->seed; us.k1 = (uint32_t)(p->seed >> 32);
    if (pos < 0) return fail(x, KG_EINVAL, "negative position");
    if (!p->uniforms) return KG_OK;
    if (pos >= p->n_uniform_positions) return fail(x, KG_EINVAL, "uniforms cover %d positions, position %d needed", p->n_uniform_positions, pos);
    const int pu[2] = {purpose0, purpose1};
    for (int w = 0; w < 2; w++) {
        if (pu[w] < 0) continue;
        const float u = p->uniforms[(size_t)pos * 3 + pu[w]];
        if (!(u >= 0.f && u < 1.f)) return fail(x, KG_EINVAL, "uniform number outside [0,1)");
        (w ? us.u1 : us.u0)[row] = u;
    }
    return KG_OK;
}

// a token outside the vocabulary means the logits were not finite (the arg-max found no maximum)
int check_tokens(kg_ctx *x, int n)
{
    for (int i = 0; i < n; i++)
        if (x->h_tok[i] < 0 || x->h_tok[i] >= x->c.vocab)
            return fail(x, KG_EHIP, "row %d: the LM head produced no valid token (non-finite logits)", i);
    return KG_OK;
}

int fetch_results(kg_ctx *x, int n)
{
    prof_flush(x);
    HIPCHK(x, hipMemcpyAsync(x->h_tok, x->scr + x->s_tok, KG_ROWS * 8, hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    if (x->profiling) prof_collect(x);
    return check_tokens(x, n);
}

float *Frow(kg_ctx *x, int j) { return at<float>(x->scr, x->s_F) + (size_t)(j + 1) * x->c.d_model; } // f_j
float *Flag(kg_ctx *x) { return at<float>(x->scr, x->s_F); }

// shallow sub-network M^b[:l] on M tokens at pos0; early features go to rows f_j0..f_{j0+M-1}
int run_shallow(kg_ctx *x, const int *tokens, int M, int pos0, int j0, const int *tok_dev = nullptr)
{
    const kg_config &c = x->c;
    float *x0 = at<float>(x->scr, x->s_x0);
    KGCHK(launch_pack_rows(x, tokens, nullptr, M, at<const float>(x->arena, x->lw[0].g1), x0, x->scr + x->s_actX,
                           at<float>(x->scr, x->s_ssq0), tok_dev));
    return run_layers(x, 0, c.exit_layer, M, pos0, x0, Frow(x, j0), nullptr);
}

// adapter A on rows starting at F-buffer row `frow` (0 = lag slot), positions pos0..; when
// `full` is false only its K/V are appended (prefill).  Leaves actX/ssq0 ready for the LM head.
int run_adapter(kg_ctx *x, int frow, int M, int pos0, bool full)
{
    const kg_config &c = x->c;
    const int d = c.d_model;
    const float *rows = at<float>(x->scr, x->s_F) + (size_t)frow * c.d_model;
    const float *glast = at<const float>(x->arena, x->a_glast);
    if (x->akind == KG_ADAPTER_MLP && !full) return KG_OK;      // no cache to fill
    KGCHK(launch_pack_rows(x, nullptr, rows, M, at<const float>(x->arena, x->a_gin), nullptr, x->scr + x->s_actX,
                           at<float>(x->scr, x->s_ssq0)));
    if (x->akind == KG_ADAPTER_MLP) {
        // h = f + W2 . silu(W1 . RMSNorm(f; g_in)), then the last norm is folded into the head's input
        Epi e = epi_base(x, EPI_SILU, M, d);
        e.ssq_in = at<float>(x->scr, x->s_ssq0); e.act_out = x->scr + x->s_actA; e.act_K = d;
        KGCHK(launch_gemv(x, x->a_w1, d, d, x->scr + x->s_actX, e));
        e = epi_base(x, EPI_RESID, M, d);
        e.res = rows; e.xout = at<float>(x->scr, x->s_x1); e.act_out = x->scr + x->s_actX; e.act_K = d;
        e.gain = glast; e.ssq_out = at<float>(x->scr, x->s_ssq0);
        return launch_gemv(x, x->a_w2, d, d, x->scr + x->s_actA, e);
    }
    if (!full) {
        Epi e = epi_base(x, EPI_PLAIN, M, 3 * c.d_model);
        e.ssq_in = at<float>(x->scr, x->s_ssq0); e.out = at<float>(x->scr, x->s_qkv);
        KGCHK(launch_gemv(x, x->a_qkv, 3 * c.d_model, c.d_model, x->scr + x->s_actX, e));
        return launch_attn(x, c.n_layers, pos0, M, 1);
    }
    if (x->akind == KG_ADAPTER_LAYER)     // one whole decoder block with the adapter's weights
        return run_block(x, c.n_layers, x->a_qkv, x->a_wo, x->a_gu, x->a_wd, at<const float>(x->arena, x->a_gpost), M,
                         pos0, rows, at<float>(x->scr, x->s_x0), glast, true);
    return run_block(x, c.n_layers, x->a_qkv, x->a_wo, 0, 0, nullptr, M, pos0, rows, at<float>(x->scr, x->s_x1), glast,
                     false);
}

// remaining layers M^b[l:] on early features f_0..f_{M-1} at pos0, then final norm (folded) —
// leaves actX/ssq0 ready for the LM head.
int run_deep(kg_ctx *x, int M, int pos0)
{
    const kg_config &c = x->c;
    const float *gf = at<const float>(x->arena, x->gfinal);
    if (c.exit_layer == c.n_layers)
        return launch_pack_rows(x, nullptr, Frow(x, 0), M, gf, nullptr, x->scr + x->s_actX, at<float>(x->scr, x->s_ssq0));
    KGCHK(launch_pack_rows(x, nullptr, Frow(x, 0), M, at<const float>(x->arena, x->lw[c.exit_layer].g1), nullptr,
                           x->scr + x->s_actX, at<float>(x->scr, x->s_ssq0)));
    return run_layers(x, c.exit_layer, c.n_layers, M, pos0, Frow(x, 0), at<float>(x->scr, x->s_x0), gf);
}

int check_ready(kg_ctx *x)
{
    if (!x) return KG_EINVAL;
    if (!x->bound) return fail(x, KG_ESTATE, "kg_bind has not been called");
    for (size_t i = 0; i < x->loaded.size(); i++)
        if (!x->loaded[i]) return fail(x, KG_ESTATE, "tensor slot %zu has not been loaded", i);
    return KG_OK;
}

int check_params(kg_ctx *x, const kg_params *p)
{
    if (!p) return fail(x, KG_EINVAL, "params is NULL");
    if (p->gamma < 1 || p->gamma > x->c.gamma_max) return fail(x, KG_EINVAL, "gamma %d outside 1..%d", p->gamma, x->c.gamma_max);
    if (p->mode != 0 && p->mode != 1) return fail(x, KG_EINVAL, "mode %d is neither 0 (greedy) nor 1 (sampling)", p->mode);
    if (p->mode == 1) {
        if (!(p->temperature > 0.f)) return fail(x, KG_EINVAL, "temperature must be > 0");
        if (p->uniforms && p->n_uniform_positions < 1) return fail(x, KG_EINVAL, "empty table of uniform numbers");
    }
    if (!(p->eta >= 0.f)) return fail(x, KG_EINVAL, "eta must be >= 0");
    return KG_OK;
}

// does the context's adapter architecture (Table 2) have this adapter tensor?
bool adapter_has(const kg_ctx *x, int kind)
{
    switch (kind) {
    case KG_A_WQ: case KG_A_WK: case KG_A_WV: case KG_A_WO: return x->akind != KG_ADAPTER_MLP;
    case KG_A_NORM_IN: case KG_A_NORM_LAST: return true;
    case KG_A_HEAD: return x->akind == KG_ADAPTER_ATTN_HEAD || x->akind == KG_ADAPTER_MLP;
    case KG_A_NORM_POST: case KG_A_WG: case KG_A_WU: case KG_A_WD: return x->akind == KG_ADAPTER_LAYER;
    case KG_A_W1: case KG_A_W2: return x->akind == KG_ADAPTER_MLP;
    }
    return false;
}

int tensor_slot(const kg_ctx *x, int kind, int layer)
{
    // slot index into `loaded`: 3 globals, 9 per layer, 13 adapter kinds
    if (kind <= KG_FINAL_NORM) return kind;
    if (kind <= KG_NORM2) return 3 + layer * 9 + (kind - KG_WQ);
    return 3 + x->c.n_layers * 9 + (kind - KG_A_WQ);
}

double now_s()
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

} // namespace

// ================================================================================================
extern "C" {

int kg_stats_cr(const kg_stats *st, double *cr)
{
    if (!st || !cr || st->rounds < 1) return KG_EINVAL;
    long tokens = 0, rounds = 0;
    for (int s = 0; s <= KG_MAX_ROWS; s++) { tokens += (long)s * st->s_hist[s]; rounds += st->s_hist[s]; }
    if (rounds < 1) return KG_EINVAL;
    *cr = (double)tokens / (double)rounds;
    return KG_OK;
}

int kg_stats_ctar(const kg_stats *st, int w, double *ctar)
{
    if (!st || !ctar || w < 1) return KG_EINVAL;
    long over = 0, rounds = 0;
    for (int s = 0; s <= KG_MAX_ROWS; s++) { rounds += st->s_hist[s]; if (s - w > 0) over += st->s_hist[s]; }
    if (rounds < 1) return KG_EINVAL;
    *ctar = (double)over / (double)rounds;
    return KG_OK;
}

int kg_create(const kg_config *cfg, kg_ctx **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return KG_EINVAL;
    const kg_config &c = *cfg;
    if (c.n_layers < 1 || c.d_model < 16 || c.n_heads < 1 || c.d_ffn < 8 || c.vocab < 16) return KG_EINVAL;
    if (c.head_dim != 64 && c.head_dim != 128) return KG_EINVAL;
    if (c.n_heads * c.head_dim != c.d_model) return KG_EINVAL;
    if (c.d_model % 16 || c.d_ffn % 8 || c.vocab % 16 || c.d_model > 8192) return KG_EINVAL;
    if (c.exit_layer < 1 || c.exit_layer > c.n_layers) return KG_EINVAL;
    if (c.dtype != 0 && c.dtype != 1) return KG_EINVAL;
    if (c.kv_dtype < 0 || c.kv_dtype > 2) return KG_EINVAL;
    if (c.dtype == 0 && c.kv_dtype != 0) return KG_EINVAL;   // fp32 weights keep an fp32 cache
    if (c.gamma_max < 1 || c.gamma_max > KG_MAX_ROWS - 1) return KG_EINVAL;
    if (c.kv_page_tokens < 16 || c.kv_page_tokens > 128 || (c.kv_page_tokens & (c.kv_page_tokens - 1))) return KG_EINVAL;
    if ((c.max_seq + c.kv_page_tokens - 1) / c.kv_page_tokens > 128) return KG_EINVAL;   // at most 128 KV pages
    if (c.max_seq < 2 || !(c.rms_eps >= 0.f) || !(c.rope_theta > 0.f)) return KG_EINVAL;
    if (c.adapter_kind < KG_ADAPTER_ATTN || c.adapter_kind > KG_ADAPTER_MLP) return KG_EINVAL;
    kg_ctx *x = new (std::nothrow) kg_ctx();
    if (!x) return KG_ENOMEM;
    x->c = c;
    x->akind = c.adapter_kind;
    x->bf = c.dtype == 1;
    x->esz = x->bf ? 2 : 4;
    x->kvt = c.kv_dtype;
    x->kvesz = x->kvt ? 2 : 4;
    x->KSd = (c.d_model + 31) / 32;
    x->KSf = (c.d_ffn + 31) / 32;
    x->logP = ilog2(c.kv_page_tokens);
    x->n_pages = (c.max_seq + c.kv_page_tokens - 1) / c.kv_page_tokens;
    x->err[0] = 0;
    memset(&x->prof, 0, sizeof(x->prof));
    layout(x);
    x->loaded.assign(3 + (size_t)c.n_layers * 9 + (KG_N_TENSOR_KINDS - KG_A_WQ), 0);
    x->page_order.resize(x->n_pages);
    for (int i = 0; i < x->n_pages; i++) x->page_order[i] = i;
    *out = x;
    return KG_OK;
}

int kg_workspace_bytes(const kg_ctx *x, size_t *weight_bytes, size_t *kv_bytes, size_t *scratch_bytes)
{
    if (!x) return KG_EINVAL;
    if (weight_bytes) *weight_bytes = x->arena_bytes;
    if (kv_bytes) *kv_bytes = x->kv_bytes;
    if (scratch_bytes) *scratch_bytes = x->scratch_bytes;
    return KG_OK;
}

static int upload_tables(kg_ctx *x)
{
    const kg_config &c = x->c;
    HIPCHK(x, hipMemsetAsync(x->scr, 0, x->scratch_bytes, x->stream));
    HIPCHK(x, hipMemcpyAsync(x->scr + x->s_pt, x->page_order.data(), (size_t)x->n_pages * 4, hipMemcpyHostToDevice,
                             x->stream));
    std::vector<double> invf(c.head_dim / 2);
    for (int i = 0; i < c.head_dim / 2; i++) invf[i] = std::pow((double)c.rope_theta, -2.0 * i / c.head_dim);
    HIPCHK(x, hipMemcpyAsync(x->scr + x->s_invf, invf.data(), invf.size() * 8, hipMemcpyHostToDevice, x->stream));
    int n = c.max_seq * (c.head_dim / 2);
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, x->stream, at<float2>(x->scr, x->s_rope),
                       c.max_seq, c.head_dim / 2, at<const double>(x->scr, x->s_invf));
    KGCHK(check_launch(x, "rope_table"));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    return KG_OK;
}

int kg_bind(kg_ctx *x, void *weights_dev, size_t weight_bytes, void *kv_dev, size_t kv_bytes, void *scratch_dev,
            size_t scratch_bytes, void *hip_stream)
{
    if (!x) return KG_EINVAL;
    if (!weights_dev || !kv_dev || !scratch_dev) return fail(x, KG_EINVAL, "NULL device buffer");
    if (((uintptr_t)weights_dev | (uintptr_t)kv_dev | (uintptr_t)scratch_dev) & (ALIGN - 1))
        return fail(x, KG_EINVAL, "device buffers must be %zu-byte aligned", ALIGN);
    if (weight_bytes < x->arena_bytes || kv_bytes < x->kv_bytes || scratch_bytes < x->scratch_bytes)
        return fail(x, KG_ENOSPC, "buffers too small: need %zu/%zu/%zu bytes", x->arena_bytes, x->kv_bytes, x->scratch_bytes);
    x->arena = (char *)weights_dev; x->kv = (char *)kv_dev; x->scr = (char *)scratch_dev;
    x->stream = (hipStream_t)hip_stream;
    if (!x->h_tok) {
        HIPCHK(x, hipHostMalloc((void **)&x->h_tok, KG_ROWS * 8, hipHostMallocDefault));
        x->h_conf = reinterpret_cast<float *>(x->h_tok + KG_ROWS);
        HIPCHK(x, hipEventCreateWithFlags(&x->ev_fetch, hipEventDisableTiming));
    }
    x->bound = true;
    x->tr = nullptr;
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            x->n_cus = cus;
    }
    std::fill(x->loaded.begin(), x->loaded.end(), 0);
    for (int k = KG_A_WQ; k < KG_N_TENSOR_KINDS; k++)       // adapter tensors this architecture does not have
        if (!adapter_has(x, k)) x->loaded[tensor_slot(x, k, -1)] = 1;
    x->phase = Phase::NONE;
    return upload_tables(x);
}

int kg_load_tensor(kg_ctx *x, int kind, int layer, const void *src, size_t n_elements)
{
    if (!x) return KG_EINVAL;
    if (!x->bound) return fail(x, KG_ESTATE, "kg_bind has not been called");
    if (!src) return fail(x, KG_EINVAL, "NULL tensor");
    const kg_config &c = x->c;
    const int d = c.d_model, f = c.d_ffn, V = c.vocab;
    if (kind < 0 || kind >= KG_N_TENSOR_KINDS) return fail(x, KG_EINVAL, "unknown tensor kind %d", kind);
    bool per_layer = kind >= KG_WQ && kind <= KG_NORM2;
    if (per_layer ? (layer < 0 || layer >= c.n_layers) : (layer != -1))
        return fail(x, KG_EINVAL, "bad layer %d for tensor kind %d", layer, kind);
    if (kind >= KG_A_WQ && !adapter_has(x, kind))
        return fail(x, KG_EINVAL, "tensor kind %d is not part of adapter architecture %d", kind, x->akind);
    int rows = 0, K = 0, row_off = 0, mode = 0;
    size_t dst = 0;
    bool is_gain = false;
    switch (kind) {
    case KG_EMBED: rows = V; K = d; dst = x->embed; break;
    case KG_LM_HEAD: rows = V; K = d; dst = x->head; break;
    case KG_FINAL_NORM: is_gain = true; dst = x->gfinal; break;
    case KG_WQ: case KG_WK: case KG_WV: rows = d; K = d; dst = x->lw[layer].qkv; row_off = (kind - KG_WQ) * d; break;
    case KG_WO: rows = d; K = d; dst = x->lw[layer].wo; break;
    case KG_WG: case KG_WU: rows = f; K = d; dst = x->lw[layer].gu; mode = 1 + (kind - KG_WG); break;
    case KG_WD: rows = d; K = f; dst = x->lw[layer].wd; break;
    case KG_NORM1: is_gain = true; dst = x->lw[layer].g1; break;
    case KG_NORM2: is_gain = true; dst = x->lw[layer].g2; break;
    case KG_A_WQ: case KG_A_WK: case KG_A_WV: rows = d; K = d; dst = x->a_qkv; row_off = (kind - KG_A_WQ) * d; break;
    case KG_A_WO: rows = d; K = d; dst = x->a_wo; break;
    case KG_A_NORM_IN: is_gain = true; dst = x->a_gin; break;
    case KG_A_NORM_LAST: is_gain = true; dst = x->a_glast; break;
    case KG_A_HEAD: rows = V; K = d; dst = x->a_head; break;
    case KG_A_NORM_POST: is_gain = true; dst = x->a_gpost; break;
    case KG_A_WG: case KG_A_WU: rows = f; K = d; dst = x->a_gu; mode = 1 + (kind - KG_A_WG); break;
    case KG_A_WD: rows = d; K = f; dst = x->a_wd; break;
    case KG_A_W1: rows = d; K = d; dst = x->a_w1; break;
    case KG_A_W2: rows = d; K = d; dst = x->a_w2; break;
    }
    size_t want = is_gain ? (size_t)d : (size_t)rows * K;
    if (n_elements != want) return fail(x, KG_EINVAL, "tensor kind %d: %zu elements given, %zu expected", kind, n_elements, want);
    if (is_gain) {
        hipLaunchKernelGGL(gain_to_f32_kernel, dim3((d + 255) / 256), dim3(256), 0, x->stream, src, x->bf ? 1 : 0, d,
                           at<float>(x->arena, dst));
    } else if (kind == KG_EMBED) {
        HIPCHK(x, hipMemcpyAsync(x->arena + dst, src, want * x->esz, hipMemcpyDeviceToDevice, x->stream));
    } else if (x->bf) {
        if (K % 8) return fail(x, KG_EINVAL, "bf16 tensors need K %% 8 == 0");
        int KS = (K + 31) / 32;
        size_t total = (size_t)rows * KS * 4;
        hipLaunchKernelGGL(pack_w_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, x->stream,
                           (const uint16_t *)src, rows, K, at<u32x4_t>(x->arena, dst), KS, row_off, mode);
    } else {
        size_t total = (size_t)rows * K;
        hipLaunchKernelGGL(pack_w_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, x->stream,
                           (const float *)src, rows, K, at<float>(x->arena, dst), row_off, mode);
    }
    KGCHK(check_launch(x, "load_tensor"));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    x->loaded[tensor_slot(x, kind, layer)] = 1;
    if (kind >= KG_A_WQ) x->tr = nullptr;   // the training master copies no longer match the adapter: bind again
    return KG_OK;
}

int kg_set_page_order(kg_ctx *x, const int32_t *perm, int n)
{
    if (!x || !perm) return KG_EINVAL;
    if (n != x->n_pages) return fail(x, KG_EINVAL, "page order has %d entries, the pool has %d pages", n, x->n_pages);
    std::vector<char> seen(n, 0);
    for (int i = 0; i < n; i++) {
        if (perm[i] < 0 || perm[i] >= n || seen[perm[i]]) return fail(x, KG_EINVAL, "page order is not a permutation");
        seen[perm[i]] = 1;
    }
    x->page_order.assign(perm, perm + n);
    x->phase = Phase::NONE;
    if (x->bound) {
        HIPCHK(x, hipMemcpyAsync(x->scr + x->s_pt, x->page_order.data(), (size_t)n * 4, hipMemcpyHostToDevice, x->stream));
        HIPCHK(x, hipStreamSynchronize(x->stream));
    }
    return KG_OK;
}

int kg_reset(kg_ctx *x)
{
    if (!x) return KG_EINVAL;
    x->phase = Phase::NONE;
    x->base = x->adapter_len = x->lag = 0;
    x->n_drafts = x->stopped = 0;
    x->pending = -1;
    x->spec_shallow = -1;
    if (x->bound) {
        HIPCHK(x, hipMemsetAsync(x->scr + x->s_cnt, 0, (size_t)x->c.n_heads * 4, x->stream));
        if (x->pf_rows > 0)
            HIPCHK(x, hipMemsetAsync(x->scr + x->s_pcnt, 0, (size_t)(x->pf_rows / KG_ROWS) * x->c.n_heads * 4, x->stream));
        HIPCHK(x, hipStreamSynchronize(x->stream));
    }
    return KG_OK;
}

int kg_prefill(kg_ctx *x, const kg_params *p, const int32_t *prompt, int n, int32_t *first_token)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!prompt || !first_token || n < 1) return fail(x, KG_EINVAL, "bad prompt");
    const kg_config &c = x->c;
    if (n + 1 + p->gamma + 1 > c.max_seq) return fail(x, KG_ENOSPC, "prompt of %d tokens does not fit max_seq %d", n, c.max_seq);
    for (int i = 0; i < n; i++)
        if (prompt[i] < 0 || prompt[i] >= c.vocab) return fail(x, KG_EINVAL, "prompt token %d out of range", prompt[i]);
    USrc u_first;
    memset(&u_first, 0, sizeof(u_first));
    KGCHK(usrc_row(x, p, u_first, 0, n, 2));
    KGCHK(kg_reset(x));
    x->acct_phase = 3;
    float inv_t = p->mode == 1 ? 1.f / p->temperature : 1.f;
    if (x->pf_rows > 0) {
        // bf16 weights: the prompt goes through the MFMA projections, pf_rows rows per pass
        HIPCHK(x, hipMemcpyAsync(x->scr + x->s_ptok, prompt, (size_t)n * 4, hipMemcpyHostToDevice, x->stream));
        for (int pos0 = 0; pos0 < n; pos0 += x->pf_rows) {
            const int T = std::min(x->pf_rows, n - pos0);
            const float *x_last = nullptr;
            KGCHK(pf_rows_pass(x, pos0, T, &x_last));
            if (pos0 + T == n) {
                // target distribution of the first new token: final norm + LM head on the last row
                KGCHK(launch_pack_rows(x, nullptr, x_last + (size_t)(T - 1) * c.d_model, 1, at<const float>(x->arena, x->gfinal),
                                       nullptr, x->scr + x->s_actX, at<float>(x->scr, x->s_ssq0)));
                KGCHK(run_head(x, 1, 0, at<float>(x->scr, x->s_tlog), 1, inv_t, p->mode, &u_first, 2));
            }
        }
    } else {
        for (int pos0 = 0; pos0 < n; pos0 += KG_ROWS) {
            int M = std::min(KG_ROWS, n - pos0);
            KGCHK(run_shallow(x, prompt + pos0, M, pos0, 0));
            KGCHK(run_adapter(x, 1, M, pos0, false));
            KGCHK(run_deep(x, M, pos0));
            if (pos0 + M == n) KGCHK(run_head(x, M, -(M - 1), at<float>(x->scr, x->s_tlog), 1, inv_t, p->mode, &u_first, 2));
        }
    }
    KGCHK(fetch_results(x, 1));
    x->base = n; x->adapter_len = n; x->lag = 0;
    x->n_drafts = 0; x->stopped = 0;
    x->n_target_rows = 1;
    x->pending = x->h_tok[0];
    x->plain_len = n;
    x->phase = Phase::READY;
    *first_token = x->pending;
    return KG_OK;
}

int kg_draft_step(kg_ctx *x, const kg_params *p, int32_t *token, float *confidence, int *stop)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!token || !confidence || !stop) return fail(x, KG_EINVAL, "NULL output");
    if (x->phase != Phase::READY && x->phase != Phase::DRAFTING) return fail(x, KG_ESTATE, "draft_step needs a prefilled sequence and no pending verify");
    if (x->stopped || x->n_drafts >= p->gamma) return fail(x, KG_ESTATE, "drafting already ended for this round");
    const int j = x->n_drafts;
    if (x->base + j + 2 >= x->c.max_seq) return fail(x, KG_ENOSPC, "sequence would exceed max_seq");
    const int tok = j == 0 ? x->pending : x->drafts[j - 1];
    const int pos = x->base + j;
    USrc u_draft;
    memset(&u_draft, 0, sizeof(u_draft));
    KGCHK(usrc_row(x, p, u_draft, 0, pos + 1, 0));
    // a run-ahead pass that becomes this step's shallow pass was booked as shallow-only: move it
    x->acct_phase = 0;
    if (x->spec_shallow != j) KGCHK(run_shallow(x, &tok, 1, pos, j));
    else { x->acct[1] -= x->spec_cost; x->acct[0] += x->spec_cost; }
    x->spec_shallow = -1;
    int M = 1;
    if (j == 0 && x->lag && x->akind != KG_ADAPTER_MLP) {   // adapter catches up on [lagged f, f_0] (Figure 2)
        M = 2;
        KGCHK(run_adapter(x, 0, 2, pos - 1, true));
    } else {
        KGCHK(run_adapter(x, j + 1, 1, pos, true));
    }
    float inv_t = p->mode == 1 ? 1.f / p->temperature : 1.f;
    float *dl = at<float>(x->scr, x->s_dlog) + (size_t)j * x->c.vocab;
    KGCHK(run_head(x, M, -(M - 1), dl, 1, inv_t, p->mode, &u_draft, 0, at<float>(x->scr, x->s_dstat) + 2 * j, true));
    // The draft token's early feature is needed whatever the host decides next (one more draft
    // step, or verification): compute it now, reading the token from device memory, so that the
    // GPU keeps working while the host waits for the token and its confidence.  The results are
    // copied out first: the copy is ordered before these kernels on the stream.
    HIPCHK(x, hipMemcpyAsync(x->h_tok, x->scr + x->s_tok, KG_ROWS * 8, hipMemcpyDeviceToHost, x->stream));
    hipEvent_t ev = x->ev_fetch;
    HIPCHK(x, hipEventRecord(ev, x->stream));
    {
        x->acct_phase = 1;
        const double before = x->acct[1];
        KGCHK(run_shallow(x, nullptr, 1, pos + 1, j + 1, at<const int>(x->scr, x->s_tok)));
        x->spec_cost = x->acct[1] - before;
    }
    x->spec_shallow = j + 1;
    HIPCHK(x, hipEventSynchronize(ev));
    KGCHK(check_tokens(x, 1));
    x->lag = 0;
    x->adapter_len = pos + 1;
    x->drafts[j] = x->h_tok[0];
    x->confs[j] = x->h_conf[0];
    x->n_drafts = j + 1;
    x->stopped = (x->confs[j] < p->eta) || (x->n_drafts == p->gamma);   // Eq. 4
    x->phase = Phase::DRAFTING;
    *token = x->drafts[j];
    *confidence = x->confs[j];
    *stop = x->stopped;
    return KG_OK;
}

int kg_verify(kg_ctx *x, const kg_params *p, int32_t *target_tokens, int *k_plus_1)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!target_tokens || !k_plus_1) return fail(x, KG_EINVAL, "NULL output");
    if (x->phase != Phase::DRAFTING || x->n_drafts < 1) return fail(x, KG_ESTATE, "verify needs at least one draft step");
    const int k = x->n_drafts;
    if (x->base + k + 1 >= x->c.max_seq) return fail(x, KG_ENOSPC, "sequence would exceed max_seq");
    const int tok = x->drafts[k - 1];
    x->acct_phase = 1;
    if (x->spec_shallow != k) KGCHK(run_shallow(x, &tok, 1, x->base + k, k));   // next early feature f_k; adapter not run
    x->spec_shallow = -1;
    x->acct_phase = 2;
    KGCHK(run_deep(x, k + 1, x->base));
    float inv_t = p->mode == 1 ? 1.f / p->temperature : 1.f;
    KGCHK(run_head(x, k + 1, 0, at<float>(x->scr, x->s_tlog), k + 1, inv_t));
    KGCHK(fetch_results(x, k + 1));
    for (int i = 0; i <= k; i++) { x->targets[i] = x->h_tok[i]; target_tokens[i] = x->h_tok[i]; }
    x->n_target_rows = k + 1;
    *k_plus_1 = k + 1;
    x->phase = Phase::VERIFIED;
    return KG_OK;
}

int kg_accept(kg_ctx *x, const kg_params *p, int32_t *emitted, int *n_emitted)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!emitted || !n_emitted) return fail(x, KG_EINVAL, "NULL output");
    if (x->phase != Phase::VERIFIED) return fail(x, KG_ESTATE, "accept needs a verified round");
    const int k = x->n_drafts;
    int n = 0;
    if (p->mode == 0) {
        while (n < k && x->drafts[n] == x->targets[n]) n++;
        for (int i = 0; i < n; i++) emitted[i] = x->drafts[i];
        emitted[n] = x->targets[n];
    } else {
        I8 dr;
        USrc us;
        memset(&us, 0, sizeof(us));
        for (int i = 0; i < KG_ROWS; i++) dr.v[i] = i < k ? x->drafts[i] : 0;
        for (int i = 0; i <= k; i++)               // row i decides the token at position base + i + 1
            KGCHK(usrc_row(x, p, us, i, x->base + i + 1, i < k ? 1 : -1, 2));
        {
            ProfScope ps(x, 2, 0.0);
            hipLaunchKernelGGL(accept_sample_kernel, dim3(1), dim3(1024), 0, x->stream, at<const float>(x->scr, x->s_tlog),
                               at<const float>(x->scr, x->s_dlog), at<const float>(x->scr, x->s_tstat),
                               at<const float>(x->scr, x->s_dstat), at<const float>(x->scr, x->s_hstat), x->c.vocab, k,
                               1.f / p->temperature, dr, us,
                               at<int>(x->scr, x->s_acc));
            KGCHK(check_launch(x, "accept_sample"));
        }
        prof_flush(x);
        HIPCHK(x, hipMemcpyAsync(x->h_tok, x->scr + x->s_acc, 8, hipMemcpyDeviceToHost, x->stream));
        HIPCHK(x, hipStreamSynchronize(x->stream));
        if (x->profiling) prof_collect(x);
        n = x->h_tok[0];
        if (n < 0 || n > k) return fail(x, KG_EHIP, "acceptance kernel returned %d accepted drafts of %d", n, k);
        if (x->h_tok[1] < 0 || x->h_tok[1] >= x->c.vocab)
            return fail(x, KG_EHIP, "acceptance kernel drew no valid token (non-finite logits)");
        for (int i = 0; i < n; i++) emitted[i] = x->drafts[i];
        emitted[n] = x->h_tok[1];
    }
    *n_emitted = n + 1;
    // rollback: caches are cut by length; the adapter saw f_0..f_{k-1} only
    const int old = x->base;
    x->base = old + n + 1;
    x->adapter_len = old + std::min(n + 1, k);
    x->lag = (n == k);
    if (x->lag) {
        HIPCHK(x, hipMemcpyAsync(Flag(x), Frow(x, k), (size_t)x->c.d_model * 4, hipMemcpyDeviceToDevice, x->stream));
    }
    x->pending = emitted[n];
    x->plain_len = x->base;      // a plain step after this round continues the committed sequence
    x->n_drafts = 0; x->stopped = 0;
    x->phase = Phase::READY;
    return KG_OK;
}

int kg_generate(kg_ctx *x, const kg_params *p, const int32_t *prompt, int n_prompt, int max_new, int32_t *out,
                int *n_out, kg_stats *st)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!out || !n_out || max_new < 1) return fail(x, KG_EINVAL, "bad output arguments");
    if (n_prompt + max_new + p->gamma + 1 > x->c.max_seq) return fail(x, KG_ENOSPC, "prompt + max_new + gamma + 1 exceeds max_seq");
    kg_stats s;
    memset(&s, 0, sizeof(s));
    int32_t tok;
    KGCHK(kg_prefill(x, p, prompt, n_prompt, &tok));
    const double a0[3] = {x->acct[0], x->acct[1], x->acct[2]};
    double t0 = now_s();
    int n = 0;
    out[n++] = tok;
    while (n < max_new) {
        double ta = now_s();
        int stop = 0;
        float conf;
        while (!stop) { KGCHK(kg_draft_step(x, p, &tok, &conf, &stop)); s.draft_steps++; }
        double tb = now_s();
        int32_t tg[KG_MAX_ROWS], em[KG_MAX_ROWS];
        int kp1 = 0, ne = 0;
        KGCHK(kg_verify(x, p, tg, &kp1));
        KGCHK(kg_accept(x, p, em, &ne));
        double tc = now_s();
        s.t_draft_s += tb - ta; s.t_verify_s += tc - tb;
        s.rounds++; s.verify_calls++; s.drafted += kp1 - 1; s.accepted += ne - 1;
        int room = max_new - n;
        int take = ne < room ? ne : room;
        s.s_hist[take]++;
        for (int i = 0; i < take; i++) out[n++] = em[i];
    }
    s.emitted = n;
    s.t_total_s = now_s() - t0;
    s.bytes_draft = x->acct[0] - a0[0]; s.bytes_shallow = x->acct[1] - a0[1]; s.bytes_verify = x->acct[2] - a0[2];
    *n_out = n;
    if (st) *st = s;
    return KG_OK;
}

int kg_plain_step(kg_ctx *x, const kg_params *p, int32_t token, int32_t *next_token)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!next_token) return fail(x, KG_EINVAL, "NULL output");
    if (x->phase != Phase::READY && x->phase != Phase::PLAIN) return fail(x, KG_ESTATE, "plain_step needs a prefilled sequence");
    if (token < 0 || token >= x->c.vocab) return fail(x, KG_EINVAL, "token out of range");
    if (x->plain_len + 1 >= x->c.max_seq) return fail(x, KG_ENOSPC, "sequence would exceed max_seq");
    const kg_config &c = x->c;
    float *x0 = at<float>(x->scr, x->s_x0);
    const int tok = token;
    x->acct_phase = 2;
    KGCHK(launch_pack_rows(x, &tok, nullptr, 1, at<const float>(x->arena, x->lw[0].g1), x0, x->scr + x->s_actX,
                           at<float>(x->scr, x->s_ssq0)));
    KGCHK(run_layers(x, 0, c.n_layers, 1, x->plain_len, x0, x0, at<const float>(x->arena, x->gfinal)));
    float inv_t = p->mode == 1 ? 1.f / p->temperature : 1.f;
    USrc u_next;
    memset(&u_next, 0, sizeof(u_next));
    KGCHK(usrc_row(x, p, u_next, 0, x->plain_len + 1, 2));
    KGCHK(run_head(x, 1, 0, at<float>(x->scr, x->s_tlog), 1, inv_t, p->mode, &u_next, 2));
    KGCHK(fetch_results(x, 1));
    x->plain_len++;
    x->n_target_rows = 1;
    x->phase = Phase::PLAIN;     // the adapter cache is no longer in step: draft calls are refused
    *next_token = x->h_tok[0];
    return KG_OK;
}

int kg_decode_plain(kg_ctx *x, const kg_params *p, const int32_t *prompt, int n_prompt, int max_new, int32_t *out,
                    int *n_out, kg_stats *st)
{
    KGCHK(check_ready(x));
    KGCHK(check_params(x, p));
    if (!out || !n_out || max_new < 1) return fail(x, KG_EINVAL, "bad output arguments");
    if (n_prompt + max_new + 1 > x->c.max_seq) return fail(x, KG_ENOSPC, "prompt + max_new + 1 exceeds max_seq");
    kg_stats s;
    memset(&s, 0, sizeof(s));
    int32_t tok;
    KGCHK(kg_prefill(x, p, prompt, n_prompt, &tok));
    const double a2 = x->acct[2];
    double t0 = now_s();
    int n = 0;
    out[n++] = tok;
    while (n < max_new) {
        KGCHK(kg_plain_step(x, p, tok, &tok));
        out[n++] = tok;
        s.plain_steps++;
    }
    s.emitted = n;
    s.t_total_s = now_s() - t0;
    s.bytes_verify = x->acct[2] - a2;
    *n_out = n;
    if (st) *st = s;
    return KG_OK;
}

int kg_read_logits(kg_ctx *x, int which, int row, float *host_out)
{
    if (!x || !host_out) return KG_EINVAL;
    if (!x->bound) return fail(x, KG_ESTATE, "not bound");
    size_t off;
    if (which == 0) {
        if (row < 0 || row >= x->n_drafts) return fail(x, KG_EINVAL, "draft row %d outside 0..%d", row, x->n_drafts - 1);
        off = x->s_dlog;
    } else if (which == 1) {
        if (row < 0 || row >= x->n_target_rows) return fail(x, KG_EINVAL, "target row %d outside 0..%d", row, x->n_target_rows - 1);
        off = x->s_tlog;
    } else return fail(x, KG_EINVAL, "which must be 0 or 1");
    HIPCHK(x, hipMemcpyAsync(host_out, x->scr + off + (size_t)row * x->c.vocab * 4, (size_t)x->c.vocab * 4,
                             hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    return KG_OK;
}

int kg_read_feature(kg_ctx *x, int row, float *host_out)
{
    if (!x || !host_out) return KG_EINVAL;
    if (!x->bound) return fail(x, KG_ESTATE, "not bound");
    if (row < -1 || row >= KG_ROWS) return fail(x, KG_EINVAL, "feature row outside -1..%d", KG_ROWS - 1);
    HIPCHK(x, hipMemcpyAsync(host_out, Frow(x, row), (size_t)x->c.d_model * 4, hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    return KG_OK;
}

int kg_read_kv(kg_ctx *x, int slot, int pos, float *k_host, float *v_host)
{
    if (!x || !k_host || !v_host) return KG_EINVAL;
    if (!x->bound) return fail(x, KG_ESTATE, "not bound");
    const kg_config &c = x->c;
    if (slot < 0 || slot > c.n_layers || pos < 0 || pos >= c.max_seq) return fail(x, KG_EINVAL, "slot/pos out of range");
    float *tmp = at<float>(x->scr, x->s_misc);
    int n = c.d_model;
    if (x->kvt == 2)
        hipLaunchKernelGGL(kv_read_kernel<kvhalf_t>, dim3((n + 255) / 256), dim3(256), 0, x->stream, x->kv,
                           at<const int>(x->scr, x->s_pt), slot, c.n_layers + 1, c.n_heads, c.head_dim,
                           c.kv_page_tokens, x->logP, pos, tmp, tmp + n);
    else if (x->kvt == 1)
        hipLaunchKernelGGL(kv_read_kernel<uint16_t>, dim3((n + 255) / 256), dim3(256), 0, x->stream, x->kv,
                           at<const int>(x->scr, x->s_pt), slot, c.n_layers + 1, c.n_heads, c.head_dim,
                           c.kv_page_tokens, x->logP, pos, tmp, tmp + n);
    else
        hipLaunchKernelGGL(kv_read_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, x->stream, x->kv,
                           at<const int>(x->scr, x->s_pt), slot, c.n_layers + 1, c.n_heads, c.head_dim,
                           c.kv_page_tokens, x->logP, pos, tmp, tmp + n);
    KGCHK(check_launch(x, "kv_read"));
    HIPCHK(x, hipMemcpyAsync(k_host, tmp, (size_t)n * 4, hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipMemcpyAsync(v_host, tmp + n, (size_t)n * 4, hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    return KG_OK;
}

int kg_get_state(const kg_ctx *x, int *base, int *adapter_len, int *lag, int *n_drafts)
{
    if (!x) return KG_EINVAL;
    if (base) *base = x->base;
    if (adapter_len) *adapter_len = x->adapter_len;
    if (lag) *lag = x->lag;
    if (n_drafts) *n_drafts = x->n_drafts;
    return KG_OK;
}

int kg_set_profiling(kg_ctx *x, int on)
{
    if (!x) return KG_EINVAL;
    prof_flush(x);
    if (x->bound) HIPCHK(x, hipStreamSynchronize(x->stream));
    prof_collect(x);
    memset(&x->prof, 0, sizeof(x->prof));
    x->profiling = on != 0;
    return KG_OK;
}

int kg_get_profile(kg_ctx *x, kg_profile *out)
{
    if (!x || !out) return KG_EINVAL;
    *out = x->prof;
    return KG_OK;
}

const char *kg_last_error(const kg_ctx *x) { return x ? x->err : "NULL context"; }

void kg_destroy(kg_ctx *x)
{
    if (!x) return;
    if (x->h_tok) (void)hipHostFree(x->h_tok);
    for (hipEvent_t e : x->ev_pool) (void)hipEventDestroy(e);
    if (x->ev_fetch) (void)hipEventDestroy(x->ev_fetch);
    delete x;
}

// ---- adapter training (Eq. 3, AdamW) --------------------------------------------------------------

constexpr int TR_SPLIT_MAX = 8;

// One trainable tensor: where it sits in a parameter-sized block (float offset), its shape, whether
// AdamW decays it, and where and how the decode calls keep it in the arena.
struct TrTensor {
    size_t off;
    int rows, cols;          // gains: rows = 1
    bool decay;
    size_t arena_off;
    int arena_rows;          // rows of the arena matrix the tensor is part of (tile count of the packed form)
    int row_off, mode;       // map_row() arguments
};

// the trainable tensors of the context's adapter architecture, in the order of the parameter block
static std::vector<TrTensor> train_tensors(const kg_ctx *x)
{
    const int d = x->c.d_model, f = x->c.d_ffn, V = x->c.vocab;
    std::vector<TrTensor> v;
    size_t o = 0;
    auto mat = [&](int rows, int cols, size_t aoff, int arows, int row_off, int mode) {
        v.push_back({o, rows, cols, true, aoff, arows, row_off, mode});
        o += (size_t)rows * cols;
    };
    auto gain = [&](size_t aoff) { v.push_back({o, 1, d, false, aoff, 1, 0, 0}); o += d; };
    if (x->akind == KG_ADAPTER_MLP) {
        mat(d, d, x->a_w1, d, 0, 0);
        mat(d, d, x->a_w2, d, 0, 0);
    } else {
        mat(3 * d, d, x->a_qkv, 3 * d, 0, 0);
        mat(d, d, x->a_wo, d, 0, 0);
    }
    gain(x->a_gin);
    gain(x->a_glast);
    if (x->akind == KG_ADAPTER_ATTN_HEAD || x->akind == KG_ADAPTER_MLP) mat(V, d, x->a_head, V, 0, 0);
    if (x->akind == KG_ADAPTER_LAYER) {
        gain(x->a_gpost);
        mat(f, d, x->a_gu, 2 * f, 0, 1);
        mat(f, d, x->a_gu, 2 * f, 0, 2);
        mat(d, f, x->a_wd, d, 0, 0);
    }
    return v;
}

static void train_layout(const kg_ctx *x, int Tm, TrainLayout &t)
{
    const size_t d = x->c.d_model, f = x->c.d_ffn, V = x->c.vocab, H = x->c.n_heads, T = Tm;
    size_t o = 0;
    auto take = [&](size_t floats) { size_t r = o; o += up(floats * 4); return r; };
    const std::vector<TrTensor> ts = train_tensors(x);
    t.nparam = ts.back().off + (size_t)ts.back().rows * ts.back().cols;
    t.P = take(t.nparam); t.G = take(t.nparam); t.M = take(t.nparam); t.V = take(t.nparam);
    t.F = take(T * d); t.X = take(T * d); t.Xn = take(T * d); t.N = take(T * d); t.QKV = take(T * 3 * d);
    t.O = take(T * d); t.H = take(T * d); t.Mm = take(T * d);
    t.Z = take(T * V); t.Zt = take(T * V); t.dZ = take(T * V);
    t.rin = take(T); t.rlast = take(T); t.rfin = take(T);
    t.Pm = take(H * T * T); t.dS = take(H * T * T);
    t.dMm = take(T * d); t.dH = take(T * d); t.dO = take(T * d); t.dQKV = take(T * 3 * d); t.dN = take(T * d);
    t.loss = take(T);
    if (x->akind == KG_ADAPTER_LAYER) {          // the block's feed-forward half
        t.H1 = take(T * d); t.Bn = take(T * d); t.dB = take(T * d); t.rpost = take(T);
        t.Gt = take(T * f); t.Ut = take(T * f); t.Act = take(T * f); t.dAct = take(T * f); t.dGt = take(T * f); t.dUt = take(T * f);
    }
    // partial results of split contractions ([slices][T][<= 3d]); long sequences have enough output tiles unsplit
    t.part_floats = (size_t)TR_SPLIT_MAX * std::min<size_t>(T, 256) * 3 * d;
    t.part = take(t.part_floats);
    t.bytes = o;
}

static int train_tokens_max(const kg_ctx *x)
{
    // a row of attention weights is kept in LDS by the training attention kernels
    return std::min(TR_T_MAX, x->c.max_seq);
}

int kg_train_workspace_bytes(const kg_ctx *x, int max_tokens, size_t *bytes)
{
    if (!x || !bytes) return KG_EINVAL;
    if (max_tokens < 1 || max_tokens > train_tokens_max(x)) return KG_EINVAL;
    TrainLayout t;
    train_layout(x, max_tokens, t);
    *bytes = t.bytes;
    return KG_OK;
}

// master copy <-> the arena's form of one tensor (gains: fp32 in both; rounded to the storage type on the way back)
static int train_sync_tensor(kg_ctx *x, const TrTensor &tt, float *master, bool to_arena)
{
    const size_t n = (size_t)tt.rows * tt.cols;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (tt.rows == 1) {
        float *ar = at<float>(x->arena, tt.arena_off);
        if (!to_arena) HIPCHK(x, hipMemcpyAsync(master, ar, n * 4, hipMemcpyDeviceToDevice, x->stream));
        else if (x->bf) hipLaunchKernelGGL(tr_round_bf16_kernel, dim3(blocks), dim3(256), 0, x->stream, (const float *)master, (int)n, ar);
        else HIPCHK(x, hipMemcpyAsync(ar, master, n * 4, hipMemcpyDeviceToDevice, x->stream));
    } else if (x->bf) {
        const int KS = (tt.cols + 31) / 32;
        if (to_arena)     // columns are a multiple of 8 for every tiled matrix (checked at load), master rows 16-byte aligned
            hipLaunchKernelGGL(tr_pack_bf16_kernel, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, x->stream, (const float *)master, tt.rows, tt.cols, KS,
                               tt.row_off, tt.mode, at<uint16_t>(x->arena, tt.arena_off));
        else
            hipLaunchKernelGGL(tr_unpack_bf16_kernel, dim3(blocks), dim3(256), 0, x->stream, at<const uint16_t>(x->arena, tt.arena_off),
                               tt.rows, tt.cols, KS, tt.row_off, tt.mode, master);
    } else {
        hipLaunchKernelGGL(tr_copy_rows_f32_kernel, dim3(blocks), dim3(256), 0, x->stream, master, at<float>(x->arena, tt.arena_off),
                           tt.rows, tt.cols, tt.row_off, tt.mode, to_arena ? 1 : 0);
    }
    return check_launch(x, "train_sync_tensor");
}

int kg_train_bind(kg_ctx *x, void *work_dev, size_t bytes, int max_tokens)
{
    KGCHK(check_ready(x));
    if (max_tokens < 1 || max_tokens > train_tokens_max(x)) return fail(x, KG_EINVAL, "max_tokens %d outside 1..%d", max_tokens, train_tokens_max(x));
    if (!work_dev || ((uintptr_t)work_dev & (ALIGN - 1))) return fail(x, KG_EINVAL, "training workspace must be %zu-byte aligned", ALIGN);
    TrainLayout t;
    train_layout(x, max_tokens, t);
    if (bytes < t.bytes) return fail(x, KG_ENOSPC, "training workspace too small: need %zu bytes", t.bytes);
    x->tr = (char *)work_dev; x->tl = t; x->tr_T = max_tokens; x->tr_n = 0; x->tr_step = 0; x->tr_pending = 0;
    float *P = at<float>(x->tr, t.P);
    for (const TrTensor &tt : train_tensors(x)) KGCHK(train_sync_tensor(x, tt, P + tt.off, false));
    HIPCHK(x, hipMemsetAsync(x->tr + t.M, 0, t.nparam * 4, x->stream));
    HIPCHK(x, hipMemsetAsync(x->tr + t.V, 0, t.nparam * 4, x->stream));
    HIPCHK(x, hipMemsetAsync(x->tr + t.G, 0, t.nparam * 4, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    return KG_OK;
}

// may 4 consecutive elements along an operand's contiguous index be fetched as one 16-byte word?
static void tr_gemm_vec_flags(TrGemm &g)
{
    auto ok = [](const void *p, long s_contig, long s_other) {
        return s_contig == 1 && s_other % 4 == 0 && ((uintptr_t)p & 15) == 0;
    };
    g.a_vec = g.sak == 1 ? ok(g.A, g.sak, g.sam) : ok(g.A, g.sam, g.sak);
    g.b_vec = g.b_mode == 0 && (g.sbk == 1 ? ok(g.B, g.sbk, g.sbn) : ok(g.B, g.sbn, g.sbk));
    if (g.batch > 1) {      // every batch member must keep the alignment
        g.a_vec = g.a_vec && g.bsa % 4 == 0;
        g.b_vec = g.b_vec && g.bsb % 4 == 0;
    }
}

static int tr_gemm(kg_ctx *x, const void *A, long sam, long sak, const void *B, long sbk, long sbn, int b_mode, float *C,
                   long ldc, int M, int N, int K, int accumulate)
{
    TrGemm g;
    g.A = A; g.sam = sam; g.sak = sak; g.B = B; g.sbk = sbk; g.sbn = sbn; g.b_mode = b_mode; g.b_KS = x->KSd;
    g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.accumulate = accumulate;
    g.batch = 1; g.bsa = g.bsb = g.bsc = 0;
    tr_gemm_vec_flags(g);
    // few output tiles and a long k: slice k so that the launch has enough workgroups to fill the chip
    const int tiles = ((N + 127) / 128) * ((M + 63) / 64);
    int S = 1;
    while (S < TR_SPLIT_MAX && tiles * S < 1024 && K / (2 * S) >= 256 && (size_t)2 * S * M * N <= x->tl.part_floats) S *= 2;
    g.k_chunk = ((K + S - 1) / S + 15) / 16 * 16;
    g.part = at<float>(x->tr, x->tl.part);
    {
        ProfScope ps(x, 4, 2.0 * M * (double)N * K);
        hipLaunchKernelGGL(tr_gemm_kernel, dim3((N + 127) / 128, (M + 63) / 64, S), dim3(256), 0, x->stream, g);
    }
    KGCHK(check_launch(x, "train_gemm"));
    if (S > 1) {
        ProfScope ps(x, 2, 0.0);
        hipLaunchKernelGGL(tr_gemm_reduce_kernel, dim3((unsigned)(((size_t)M * N + 255) / 256)), dim3(256), 0, x->stream,
                           (const float *)g.part, S, M, N, C, ldc, accumulate);
        KGCHK(check_launch(x, "train_gemm_reduce"));
    }
    return KG_OK;
}

// One product per attention head in a single launch: head h reads A + h * bsa, B + h * bsb and writes C + h * bsc.
static int tr_gemm_heads(kg_ctx *x, const float *A, long sam, long sak, long bsa, const float *B, long sbk, long sbn, long bsb,
                         float *C, long ldc, long bsc, int M, int N, int K, int heads)
{
    TrGemm g;
    g.A = A; g.sam = sam; g.sak = sak; g.B = B; g.sbk = sbk; g.sbn = sbn; g.b_mode = 0; g.b_KS = 0;
    g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.accumulate = 0;
    g.batch = heads; g.bsa = bsa; g.bsb = bsb; g.bsc = bsc;
    g.k_chunk = (K + 15) / 16 * 16; g.part = nullptr;
    tr_gemm_vec_flags(g);
    if (heads == 1) { g.batch = 1; }
    ProfScope ps(x, 4, 2.0 * M * (double)N * K * heads);
    hipLaunchKernelGGL(tr_gemm_kernel, dim3((N + 127) / 128, (M + 63) / 64, heads), dim3(256), 0, x->stream, g);
    return check_launch(x, "train_gemm_heads");
}

// The three products with one weight matrix W [N][K] (row-major fp32 master copy) that the chain rule needs:
//   forward   Y[T][N] (+)= X[T][K] . W^T
//   backward  dX[T][K] (+)= dY[T][N] . W
//   gradient  dW[N][K] (+)= dY^T . X
static int tr_fwd(kg_ctx *x, const float *X, const float *W, float *Y, int T, int N, int K, int acc)
{
    return tr_gemm(x, X, K, 1, W, 1, K, 0, Y, N, T, N, K, acc);
}
static int tr_bwd(kg_ctx *x, const float *dY, const float *W, float *dX, int T, int N, int K, int acc)
{
    return tr_gemm(x, dY, N, 1, W, K, 1, 0, dX, K, T, K, N, acc);
}
static int tr_wgrad(kg_ctx *x, const float *dY, const float *X, float *dW, int T, int N, int K, int acc)
{
    return tr_gemm(x, dY, 1, N, X, K, 1, 0, dW, K, N, K, T, acc);
}

static int check_train_params(kg_ctx *x, const kg_train_params *hp)
{
    if (!hp) return fail(x, KG_EINVAL, "NULL argument");
    if (!(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps > 0.f) ||
        !(hp->weight_decay >= 0.f))
        return fail(x, KG_EINVAL, "bad AdamW parameters");
    return KG_OK;
}

// The frozen target model on a whole sequence: early features F and target logits Zt of every
// position into the training workspace.
static int train_frozen_forward(kg_ctx *x, const int32_t *tokens, int n)
{
    const kg_config &c = x->c;
    const int d = c.d_model, V = c.vocab;
    const TrainLayout &t = x->tl;
    auto f = [&](size_t off) { return at<float>(x->tr, off); };
    for (int i = 0; i < n; i++)
        if (tokens[i] < 0 || tokens[i] >= c.vocab) return fail(x, KG_EINVAL, "token %d out of range", tokens[i]);
    KGCHK(kg_reset(x));
    if (x->pf_rows > 0) {
        HIPCHK(x, hipMemcpyAsync(x->scr + x->s_ptok, tokens, (size_t)n * 4, hipMemcpyHostToDevice, x->stream));
        for (int pos0 = 0; pos0 < n; pos0 += x->pf_rows) {
            const int T = std::min(x->pf_rows, n - pos0);
            const float *x_last = nullptr;
            KGCHK(pf_rows_pass(x, pos0, T, &x_last));
            HIPCHK(x, hipMemcpyAsync(f(t.F) + (size_t)pos0 * d, x->scr + x->s_pF, (size_t)T * d * 4, hipMemcpyDeviceToDevice, x->stream));
            HIPCHK(x, hipMemcpyAsync(f(t.X) + (size_t)pos0 * d, x_last, (size_t)T * d * 4, hipMemcpyDeviceToDevice, x->stream));
        }
    } else {
        for (int pos0 = 0; pos0 < n; pos0 += KG_ROWS) {
            const int M = std::min(KG_ROWS, n - pos0);
            KGCHK(run_shallow(x, tokens + pos0, M, pos0, 0));
            HIPCHK(x, hipMemcpyAsync(f(t.F) + (size_t)pos0 * d, Frow(x, 0), (size_t)M * d * 4, hipMemcpyDeviceToDevice, x->stream));
            KGCHK(run_deep(x, M, pos0));
            const float *xl = c.exit_layer == c.n_layers ? Frow(x, 0) : at<const float>(x->scr, x->s_x0);
            HIPCHK(x, hipMemcpyAsync(f(t.X) + (size_t)pos0 * d, xl, (size_t)M * d * 4, hipMemcpyDeviceToDevice, x->stream));
        }
    }
    // target logits of every position: Zt = RMSNorm(X; g_final) . head^T
    {
        ProfScope ps(x, 2, 0.0);
        hipLaunchKernelGGL(tr_rmsnorm_kernel, dim3(n), dim3(256), 0, x->stream, (const float *)f(t.X), at<const float>(x->arena, x->gfinal),
                           d, c.rms_eps, f(t.Xn), f(t.rfin));
        KGCHK(check_launch(x, "train_rmsnorm"));
    }
    return tr_gemm(x, f(t.Xn), d, 1, x->arena + x->head, 1, d, x->bf ? 1 : 0, f(t.Zt), V, n, V, d, 0);
}

static int train_graph(kg_ctx *x, int n, double *loss);

int kg_train_accumulate(kg_ctx *x, const int32_t *tokens, int n, double *loss)
{
    KGCHK(check_ready(x));
    if (!x->tr) return fail(x, KG_ESTATE, "kg_train_bind has not been called");
    if (!tokens || !loss) return fail(x, KG_EINVAL, "NULL argument");
    if (n < 1 || n > x->tr_T) return fail(x, KG_EINVAL, "%d tokens outside 1..%d", n, x->tr_T);
    KGCHK(train_frozen_forward(x, tokens, n));
    return train_graph(x, n, loss);
}

int kg_train_features(kg_ctx *x, const int32_t *tokens, int n, float *F_dev, float *Zt_dev)
{
    KGCHK(check_ready(x));
    if (!x->tr) return fail(x, KG_ESTATE, "kg_train_bind has not been called");
    if (!tokens || !F_dev || !Zt_dev) return fail(x, KG_EINVAL, "NULL argument");
    if (n < 1 || n > x->tr_T) return fail(x, KG_EINVAL, "%d tokens outside 1..%d", n, x->tr_T);
    KGCHK(train_frozen_forward(x, tokens, n));
    const TrainLayout &t = x->tl;
    HIPCHK(x, hipMemcpyAsync(F_dev, x->tr + t.F, (size_t)n * x->c.d_model * 4, hipMemcpyDeviceToDevice, x->stream));
    HIPCHK(x, hipMemcpyAsync(Zt_dev, x->tr + t.Zt, (size_t)n * x->c.vocab * 4, hipMemcpyDeviceToDevice, x->stream));
    prof_flush(x);
    HIPCHK(x, hipStreamSynchronize(x->stream));
    if (x->profiling) prof_collect(x);
    x->phase = Phase::NONE;
    return KG_OK;
}

int kg_train_accumulate_features(kg_ctx *x, const float *F_dev, const float *Zt_dev, int n, double *loss)
{
    KGCHK(check_ready(x));
    if (!x->tr) return fail(x, KG_ESTATE, "kg_train_bind has not been called");
    if (!F_dev || !Zt_dev || !loss) return fail(x, KG_EINVAL, "NULL argument");
    if (n < 1 || n > x->tr_T) return fail(x, KG_EINVAL, "%d tokens outside 1..%d", n, x->tr_T);
    const TrainLayout &t = x->tl;
    HIPCHK(x, hipMemcpyAsync(x->tr + t.F, F_dev, (size_t)n * x->c.d_model * 4, hipMemcpyDeviceToDevice, x->stream));
    HIPCHK(x, hipMemcpyAsync(x->tr + t.Zt, Zt_dev, (size_t)n * x->c.vocab * 4, hipMemcpyDeviceToDevice, x->stream));
    return train_graph(x, n, loss);
}

// The adapter's forward over all n positions from the workspace's F and Zt, Eq. 3, and the backward
// pass into the gradient block (added to it when sequences are pending).
static int train_graph(kg_ctx *x, int n, double *loss)
{
    const kg_config &c = x->c;
    const int acc = x->tr_pending > 0 ? 1 : 0;     // add to the gradient block, or start it
    const int d = c.d_model, ff = c.d_ffn, V = c.vocab, H = c.n_heads, hd = c.head_dim;
    const int kind = x->akind;
    const bool own_head = kind == KG_ADAPTER_ATTN_HEAD || kind == KG_ADAPTER_MLP;
    const TrainLayout &t = x->tl;
    auto f = [&](size_t off) { return at<float>(x->tr, off); };
    // the tensors of the parameter block and of the gradient block, by role
    float *P = f(t.P), *G = f(t.G);
    const std::vector<TrTensor> ts = train_tensors(x);
    size_t o_a = ts[0].off, o_b = ts[1].off, o_gin = ts[2].off, o_glast = ts[3].off, o_head = 0, o_gpost = 0, o_wg = 0, o_wu = 0, o_wd = 0;
    if (own_head) o_head = ts[4].off;
    if (kind == KG_ADAPTER_LAYER) { o_gpost = ts[4].off; o_wg = ts[5].off; o_wu = ts[6].off; o_wd = ts[7].off; }
    const void *head = x->arena + x->head;
    const int hm_nt = x->bf ? 1 : 0, hm_nn = x->bf ? 2 : 0;
    auto other = [&]() { ProfScope ps(x, 2, 0.0); };      // timing class of everything that is not a contraction
    auto rms = [&](const float *in, const float *g, float *out, float *r) {
        other();
        hipLaunchKernelGGL(tr_rmsnorm_kernel, dim3(n), dim3(256), 0, x->stream, in, g, d, c.rms_eps, out, r);
        return check_launch(x, "train_rmsnorm");
    };
    auto rms_bwd = [&](const float *in, const float *g, const float *r, const float *dy, float *dx, float *dg) {
        other();
        hipLaunchKernelGGL(tr_rmsnorm_bwd_kernel, dim3(n), dim3(256), 0, x->stream, in, g, r, dy, d, dx);
        hipLaunchKernelGGL(tr_gain_grad_kernel, dim3((d + 63) / 64), dim3(1024), 0, x->stream, in, r, dy, n, d, dg, acc);
        return check_launch(x, "train_rmsnorm_bwd");
    };
    auto ew_blocks = [](size_t cnt) { return dim3((unsigned)((cnt + 255) / 256)); };
    const size_t nd = (size_t)n * d, nf = (size_t)n * ff;
    // ---- adapter forward over all positions
    KGCHK(rms(f(t.F), P + o_gin, f(t.N), f(t.rin)));
    HIPCHK(x, hipMemcpyAsync(f(t.H), f(t.F), nd * 4, hipMemcpyDeviceToDevice, x->stream));
    const size_t nrope = (size_t)n * (d / hd) * (hd / 2) * 2;
    if (kind == KG_ADAPTER_MLP) {
        // h = f + W2 . silu(W1 . n): U1 in QKV's first [n][d], S1 in O
        KGCHK(tr_fwd(x, f(t.N), P + o_a, f(t.QKV), n, d, d, 0));
        other();
        hipLaunchKernelGGL(tr_silu_kernel, ew_blocks(nd), dim3(256), 0, x->stream, (const float *)f(t.QKV), nd, f(t.O));
        KGCHK(check_launch(x, "train_silu"));
        KGCHK(tr_fwd(x, f(t.O), P + o_b, f(t.H), n, d, d, 1));
    } else {
        KGCHK(tr_fwd(x, f(t.N), P + o_a, f(t.QKV), n, 3 * d, d, 0));
        other();
        hipLaunchKernelGGL(tr_rope_kernel, dim3((unsigned)((nrope + 255) / 256)), dim3(256), 0, x->stream, f(t.QKV), n, d, hd,
                           at<const float2>(x->scr, x->s_rope), 0);
        KGCHK(check_launch(x, "train_rope"));
        {
            // causal attention, one product per head: S = Q.K^T, P = softmax(S / sqrt(hd)), O = P.V
            const float *Q = f(t.QKV), *K = f(t.QKV) + d, *Vv = f(t.QKV) + 2 * d;
            const long TT = (long)n * n;
            KGCHK(tr_gemm_heads(x, Q, 3 * d, 1, hd, K, 1, 3 * d, hd, f(t.Pm), n, TT, n, n, hd, H));
            other();
            hipLaunchKernelGGL(tr_softmax_causal_kernel, dim3(n, H), dim3(256), 0, x->stream, f(t.Pm), n, 1.f / sqrtf((float)hd));
            KGCHK(check_launch(x, "train_softmax"));
            KGCHK(tr_gemm_heads(x, f(t.Pm), n, 1, TT, Vv, 3 * d, 1, hd, f(t.O), d, hd, n, hd, n, H));
        }
        KGCHK(tr_fwd(x, f(t.O), P + o_b, f(t.H), n, d, d, 1));
        if (kind == KG_ADAPTER_LAYER) {
            // h <- h + Wd (silu(Wg b) * (Wu b)), b = RMSNorm(h; g_post); the attention's output h is kept in H1
            HIPCHK(x, hipMemcpyAsync(f(t.H1), f(t.H), nd * 4, hipMemcpyDeviceToDevice, x->stream));
            KGCHK(rms(f(t.H1), P + o_gpost, f(t.Bn), f(t.rpost)));
            KGCHK(tr_fwd(x, f(t.Bn), P + o_wg, f(t.Gt), n, ff, d, 0));
            KGCHK(tr_fwd(x, f(t.Bn), P + o_wu, f(t.Ut), n, ff, d, 0));
            other();
            hipLaunchKernelGGL(tr_swiglu_kernel, ew_blocks(nf), dim3(256), 0, x->stream, (const float *)f(t.Gt), (const float *)f(t.Ut), nf,
                               f(t.Act));
            KGCHK(check_launch(x, "train_swiglu"));
            KGCHK(tr_fwd(x, f(t.Act), P + o_wd, f(t.H), n, d, ff, 1));
        }
    }
    KGCHK(rms(f(t.H), P + o_glast, f(t.Mm), f(t.rlast)));
    if (own_head) KGCHK(tr_fwd(x, f(t.Mm), P + o_head, f(t.Z), n, V, d, 0));
    else KGCHK(tr_gemm(x, f(t.Mm), d, 1, head, 1, d, hm_nt, f(t.Z), V, n, V, d, 0));
    // Eq. 3 and its gradient with respect to the draft logits
    other();
    hipLaunchKernelGGL(tr_loss_kernel, dim3(n), dim3(256), 0, x->stream, (const float *)f(t.Z), (const float *)f(t.Zt), V, f(t.dZ),
                       f(t.loss));
    KGCHK(check_launch(x, "train_loss"));
    // ---- backward
    if (own_head) {
        KGCHK(tr_wgrad(x, f(t.dZ), f(t.Mm), G + o_head, n, V, d, acc));
        KGCHK(tr_bwd(x, f(t.dZ), P + o_head, f(t.dMm), n, V, d, 0));
    } else {
        KGCHK(tr_gemm(x, f(t.dZ), V, 1, head, d, 1, hm_nn, f(t.dMm), d, n, d, V, 0));
    }
    KGCHK(rms_bwd(f(t.H), P + o_glast, f(t.rlast), f(t.dMm), f(t.dH), G + o_glast));
    if (kind == KG_ADAPTER_MLP) {
        KGCHK(tr_wgrad(x, f(t.dH), f(t.O), G + o_b, n, d, d, acc));                 // dW2 = dH^T . S1
        KGCHK(tr_bwd(x, f(t.dH), P + o_b, f(t.dO), n, d, d, 0));                    // dS1 = dH . W2
        other();
        hipLaunchKernelGGL(tr_silu_bwd_kernel, ew_blocks(nd), dim3(256), 0, x->stream, (const float *)f(t.QKV), (const float *)f(t.dO), nd,
                           f(t.dQKV));
        KGCHK(check_launch(x, "train_silu_bwd"));
        KGCHK(tr_wgrad(x, f(t.dQKV), f(t.N), G + o_a, n, d, d, acc));               // dW1 = dU1^T . N
        KGCHK(tr_bwd(x, f(t.dQKV), P + o_a, f(t.dN), n, d, d, 0));                  // dN = dU1 . W1
    } else {
        if (kind == KG_ADAPTER_LAYER) {
            KGCHK(tr_wgrad(x, f(t.dH), f(t.Act), G + o_wd, n, d, ff, acc));         // dWd = dH^T . Act
            KGCHK(tr_bwd(x, f(t.dH), P + o_wd, f(t.dAct), n, d, ff, 0));            // dAct = dH . Wd
            other();
            hipLaunchKernelGGL(tr_swiglu_bwd_kernel, ew_blocks(nf), dim3(256), 0, x->stream, (const float *)f(t.Gt), (const float *)f(t.Ut),
                               (const float *)f(t.dAct), nf, f(t.dGt), f(t.dUt));
            KGCHK(check_launch(x, "train_swiglu_bwd"));
            KGCHK(tr_wgrad(x, f(t.dGt), f(t.Bn), G + o_wg, n, ff, d, acc));
            KGCHK(tr_wgrad(x, f(t.dUt), f(t.Bn), G + o_wu, n, ff, d, acc));
            KGCHK(tr_bwd(x, f(t.dGt), P + o_wg, f(t.dB), n, ff, d, 0));
            KGCHK(tr_bwd(x, f(t.dUt), P + o_wu, f(t.dB), n, ff, d, 1));
            KGCHK(rms_bwd(f(t.H1), P + o_gpost, f(t.rpost), f(t.dB), f(t.dO), G + o_gpost));   // dO is free here: d(norm input)
            other();
            hipLaunchKernelGGL(tr_add_kernel, ew_blocks(nd), dim3(256), 0, x->stream, f(t.dH), (const float *)f(t.dO), nd);   // dH1
            KGCHK(check_launch(x, "train_add"));
        }
        KGCHK(tr_wgrad(x, f(t.dH), f(t.O), G + o_b, n, d, d, acc));                 // dWo = dH^T . O
        KGCHK(tr_bwd(x, f(t.dH), P + o_b, f(t.dO), n, d, d, 0));                    // dO = dH . Wo
        {
            // dP = dO.V^T, dV = P^T.dO, dS = P (dP - rowsum(dP P)) / sqrt(hd), dQ = dS.K, dK = dS^T.Q, per head
            const float *Q = f(t.QKV), *K = f(t.QKV) + d, *Vv = f(t.QKV) + 2 * d;
            const long TT = (long)n * n;
            KGCHK(tr_gemm_heads(x, f(t.dO), d, 1, hd, Vv, 1, 3 * d, hd, f(t.dS), n, TT, n, n, hd, H));
            KGCHK(tr_gemm_heads(x, f(t.Pm), 1, n, TT, f(t.dO), d, 1, hd, f(t.dQKV) + 2 * d, 3 * d, hd, n, hd, n, H));
            other();
            hipLaunchKernelGGL(tr_dsoftmax_kernel, dim3(n, H), dim3(256), 0, x->stream, (const float *)f(t.Pm), f(t.dS), n,
                               1.f / sqrtf((float)hd));
            KGCHK(check_launch(x, "train_dsoftmax"));
            KGCHK(tr_gemm_heads(x, f(t.dS), n, 1, TT, K, 3 * d, 1, hd, f(t.dQKV), 3 * d, hd, n, hd, n, H));
            KGCHK(tr_gemm_heads(x, f(t.dS), 1, n, TT, Q, 3 * d, 1, hd, f(t.dQKV) + d, 3 * d, hd, n, hd, n, H));
        }
        other();
        hipLaunchKernelGGL(tr_rope_kernel, dim3((unsigned)((nrope + 255) / 256)), dim3(256), 0, x->stream, f(t.dQKV), n, d, hd,
                           at<const float2>(x->scr, x->s_rope), 1);
        KGCHK(check_launch(x, "train_attn_bwd"));
        KGCHK(tr_wgrad(x, f(t.dQKV), f(t.N), G + o_a, n, 3 * d, d, acc));           // dWqkv = dQKV^T . N
        KGCHK(tr_bwd(x, f(t.dQKV), P + o_a, f(t.dN), n, 3 * d, d, 0));              // dN = dQKV . Wqkv
    }
    other();
    hipLaunchKernelGGL(tr_gain_grad_kernel, dim3((d + 63) / 64), dim3(1024), 0, x->stream, (const float *)f(t.F),
                       (const float *)f(t.rin), (const float *)f(t.dN), n, d, G + o_gin, acc);
    KGCHK(check_launch(x, "train_gain_grad"));
    // loss of this sequence (before any update), summed over positions in double on the host
    std::vector<float> rows(n);
    prof_flush(x);
    HIPCHK(x, hipMemcpyAsync(rows.data(), f(t.loss), (size_t)n * 4, hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    if (x->profiling) prof_collect(x);
    double L = 0.0;
    for (int i = 0; i < n; i++) L += rows[i];
    *loss = L;
    x->tr_n = n;
    x->tr_pending++;
    x->phase = Phase::NONE;
    return KG_OK;
}

int kg_train_apply(kg_ctx *x, const kg_train_params *hp)
{
    KGCHK(check_ready(x));
    if (!x->tr) return fail(x, KG_ESTATE, "kg_train_bind has not been called");
    KGCHK(check_train_params(x, hp));
    if (x->tr_pending < 1) return fail(x, KG_ESTATE, "no gradient has been accumulated");
    const TrainLayout &t = x->tl;
    float *P = at<float>(x->tr, t.P), *G = at<float>(x->tr, t.G), *Mo = at<float>(x->tr, t.M), *Vo = at<float>(x->tr, t.V);
    // AdamW on the fp32 master copies, then the copies the decode calls read are refreshed
    x->tr_step++;
    const float c1 = (float)(1.0 - std::pow((double)hp->beta1, (double)x->tr_step));
    const float c2 = (float)(1.0 - std::pow((double)hp->beta2, (double)x->tr_step));
    { ProfScope ps(x, 2, 0.0); }
    for (const TrTensor &tt : train_tensors(x)) {
        const size_t cnt = (size_t)tt.rows * tt.cols;
        hipLaunchKernelGGL(tr_adamw_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, x->stream, P + tt.off,
                           (const float *)(G + tt.off), Mo + tt.off, Vo + tt.off, cnt, hp->lr, hp->beta1, hp->beta2, hp->eps,
                           tt.decay ? hp->weight_decay : 0.f, c1, c2);
        KGCHK(check_launch(x, "train_adamw"));
        KGCHK(train_sync_tensor(x, tt, P + tt.off, true));
    }
    prof_flush(x);
    HIPCHK(x, hipStreamSynchronize(x->stream));
    if (x->profiling) prof_collect(x);
    x->tr_pending = 0;
    x->phase = Phase::NONE;
    return KG_OK;
}

int kg_train_step(kg_ctx *x, const kg_train_params *hp, const int32_t *tokens, int n, double *loss)
{
    if (!x) return KG_EINVAL;
    KGCHK(check_train_params(x, hp));
    // a step starts from its own gradient; a call that is refused leaves what was accumulated alone
    KGCHK(check_ready(x));
    if (!x->tr) return fail(x, KG_ESTATE, "kg_train_bind has not been called");
    if (!tokens || !loss) return fail(x, KG_EINVAL, "NULL argument");
    if (n < 1 || n > x->tr_T) return fail(x, KG_EINVAL, "%d tokens outside 1..%d", n, x->tr_T);
    x->tr_pending = 0;
    KGCHK(kg_train_accumulate(x, tokens, n, loss));
    return kg_train_apply(x, hp);
}

int kg_train_read(kg_ctx *x, int what, float *host_out, size_t n_floats)
{
    if (!x || !host_out) return KG_EINVAL;
    if (!x->tr) return fail(x, KG_ESTATE, "kg_train_bind has not been called");
    const TrainLayout &t = x->tl;
    const size_t n = x->tr_n, d = x->c.d_model, V = x->c.vocab;
    size_t off = 0, cnt = 0;
    switch (what) {
    case KG_TRAIN_FEATURES: off = t.F; cnt = n * d; break;
    case KG_TRAIN_TARGET_LOGITS: off = t.Zt; cnt = n * V; break;
    case KG_TRAIN_DRAFT_LOGITS: off = t.Z; cnt = n * V; break;
    case KG_TRAIN_GRADIENTS: off = t.G; cnt = t.nparam; break;
    case KG_TRAIN_PARAMETERS: off = t.P; cnt = t.nparam; break;
    case KG_TRAIN_ROW_LOSSES: off = t.loss; cnt = n; break;
    default: return fail(x, KG_EINVAL, "unknown training buffer %d", what);
    }
    if (what != KG_TRAIN_PARAMETERS && n == 0) return fail(x, KG_ESTATE, "no training step has run");
    if (n_floats != cnt) return fail(x, KG_EINVAL, "buffer %d holds %zu floats, %zu asked", what, cnt, n_floats);
    HIPCHK(x, hipMemcpyAsync(host_out, x->tr + off, cnt * 4, hipMemcpyDeviceToHost, x->stream));
    HIPCHK(x, hipStreamSynchronize(x->stream));
    return KG_OK;
}

int kg_op_gemm_f32(const float *A, long sam, long sak, const float *B, long sbk, long sbn, float *C, long ldc, int M, int N, int K,
                   int accumulate, void *hip_stream)
{
    if (!A || !B || !C || M < 1 || N < 1 || K < 1 || ldc < N) return KG_EINVAL;
    TrGemm g;
    g.A = A; g.sam = sam; g.sak = sak; g.B = B; g.sbk = sbk; g.sbn = sbn; g.b_mode = 0; g.b_KS = 0;
    g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K; g.accumulate = accumulate;
    g.k_chunk = (K + 15) / 16 * 16; g.part = nullptr;
    g.batch = 1; g.bsa = g.bsb = g.bsc = 0;
    tr_gemm_vec_flags(g);
    hipLaunchKernelGGL(tr_gemm_kernel, dim3((N + 127) / 128, (M + 63) / 64, 1), dim3(256), 0, (hipStream_t)hip_stream, g);
    return hipGetLastError() == hipSuccess ? KG_OK : KG_EHIP;
}

// ---- stand-alone projection ---------------------------------------------------------------------

size_t kg_op_packed_bytes(int dtype, int N, int K) { return packed_bytes(dtype == 1, N, K); }
int kg_op_tile_pos(int ks, int KS)
{
    if (KS < 1 || ks < 0 || ks >= KS) return -1;
    return tile_pos(ks, KS);
}

size_t kg_op_work_bytes(int K) { return up(act_bytes(K)) ; }

int kg_op_pack(int dtype, const void *src, int N, int K, void *packed, void *hip_stream)
{
    if (!src || !packed || N < 16 || N % 16 || K < 8 || K % 8 || (dtype != 0 && dtype != 1)) return KG_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == 1) {
        int KS = (K + 31) / 32;
        size_t total = (size_t)N * KS * 4;
        hipLaunchKernelGGL(pack_w_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const uint16_t *)src, N, K, (u32x4_t *)packed, KS, 0, 0);
    } else {
        size_t total = (size_t)N * K;
        hipLaunchKernelGGL(pack_w_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const float *)src, N, K, (float *)packed, 0, 0);
    }
    return hipGetLastError() == hipSuccess ? KG_OK : KG_EHIP;
}

// Both entry points of the stand-alone projection: the activation staging area `work` comes from the
// caller (cleared with a memset) or is the library's static array (cleared by a fill kernel, which a
// stream capture can record).
static int op_linear_launch(int dtype, const void *packed, int N, int K, const float *xd, int M, float *yd, void *work,
                            hipStream_t s, bool clear_by_kernel)
{
    Tok8 tk;
    memset(&tk, 0, sizeof(tk));
    Epi e;
    memset(&e, 0, sizeof(e));
    e.kind = EPI_PLAIN; e.M = M; e.N = N; e.out = yd;
    if (dtype == 1) {
        if (clear_by_kernel) {
            const unsigned n16 = (unsigned)(act_bytes(K) / 16);
            hipLaunchKernelGGL(fill_zero_kernel, dim3((n16 + 255) / 256), dim3(256), 0, s, (u32x4_t *)work, n16);
        } else if (hipMemsetAsync(work, 0, act_bytes(K), s) != hipSuccess) return KG_EHIP;
        hipLaunchKernelGGL(pack_rows_kernel<true>, dim3(K / 16), dim3(128), 0, s, (const void *)nullptr, tk, (const int *)nullptr, xd, K, M,
                           (const float *)nullptr, (float *)nullptr, work, (float *)nullptr);
        hipLaunchKernelGGL(gemv_bf16_kernel, dim3(N / 16), dim3(64 * GEMV_WAVES), 0, s, (const u32x4_t *)packed, (K + 31) / 32,
                           e.M, (const u32x4_t *)work, e.ssq_in, e.nt_in, e.N, (const float *)nullptr, e.gain, e);
    } else {
        hipLaunchKernelGGL(pack_rows_kernel<false>, dim3(K / 16), dim3(128), 0, s, (const void *)nullptr, tk, (const int *)nullptr, xd, K, M,
                           (const float *)nullptr, (float *)nullptr, work, (float *)nullptr);
        hipLaunchKernelGGL(gemv_f32_kernel, dim3(N / 16), dim3(256), 0, s, (const float *)packed, K, (const float *)work, e);
    }
    return hipGetLastError() == hipSuccess ? KG_OK : KG_EHIP;
}

static bool op_linear_args_ok(int dtype, const void *packed, int N, int K, const float *xd, int M, const float *yd)
{
    return packed && xd && yd && N >= 16 && N % 16 == 0 && K >= 16 && K % 16 == 0 && M >= 1 && M <= KG_ROWS &&
           (dtype == 0 || dtype == 1);
}

int kg_op_linear(int dtype, const void *packed, int N, int K, const float *xd, int M, float *yd, void *work,
                 void *hip_stream)
{
    if (!op_linear_args_ok(dtype, packed, N, K, xd, M, yd) || !work) return KG_EINVAL;
    return op_linear_launch(dtype, packed, N, K, xd, M, yd, work, (hipStream_t)hip_stream, false);
}

int kg_op_linear_valu(const void *packed, int N, int K, const float *xd, float *yd, void *hip_stream)
{
    if (!packed || !xd || !yd || N < 16 || N % 16 || K < 16 || K % 16) return KG_EINVAL;
    hipLaunchKernelGGL(gemv_bf16_valu_kernel, dim3(N / 16), dim3(64 * GEMV_WAVES), 0, (hipStream_t)hip_stream,
                       (const u32x4_t *)packed, (K + 31) / 32, xd, K, yd);
    return hipGetLastError() == hipSuccess ? KG_OK : KG_EHIP;
}

// The staging area of kg_op_linear_static: one array per GPU, held until the process ends.  Host code
// never uses the array's name as an address: the device address is asked for once per device.
static __device__ __align__(256) unsigned char scratch[KG_OP_STATIC_MAX_K * KG_ROWS * 4];
static_assert(sizeof(scratch) >= (size_t)KG_OP_STATIC_MAX_K / 32 * 1024, "bf16 staging fits");
static std::mutex static_scratch_lock;
static void *static_scratch_ptr[KG_OP_STATIC_MAX_DEVICES];      // per device, NULL until first use

int kg_op_linear_static(int dtype, const void *packed, int N, int K, const float *xd, int M, float *yd, void *hip_stream)
{
    if (!op_linear_args_ok(dtype, packed, N, K, xd, M, yd)) return KG_EINVAL;
    if (K > KG_OP_STATIC_MAX_K) return KG_ENOSPC;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return KG_EHIP;
    if (dev < 0 || dev >= KG_OP_STATIC_MAX_DEVICES) return KG_EINVAL;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> g(static_scratch_lock);
        if (!static_scratch_ptr[dev]) {
            void *q = nullptr;
            if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return KG_EHIP;
            static_scratch_ptr[dev] = q;
        }
        ptr = static_scratch_ptr[dev];
    }
    return op_linear_launch(dtype, packed, N, K, xd, M, yd, ptr, (hipStream_t)hip_stream, true);
}

int kg_op_philox_words(uint64_t seed, uint32_t pos0, uint32_t purpose, int n, uint32_t *out_dev, void *hip_stream)
{
    if (!out_dev || n < 1) return KG_EINVAL;
    hipLaunchKernelGGL(philox_words_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, (uint32_t)seed,
                       (uint32_t)(seed >> 32), pos0, purpose, n, out_dev);
    return hipGetLastError() == hipSuccess ? KG_OK : KG_EHIP;
}

int kg_op_stream_read(const void *src, size_t bytes, void *work, void *hip_stream)
{
    if (!src || !work || bytes < 16 || ((uintptr_t)src & 15)) return KG_EINVAL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return KG_EHIP;
    const int grid = std::max(1, std::min(2 * cus, 1024));       // work holds 1024 words
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(512), 0, (hipStream_t)hip_stream, (const u32x4_t *)src, bytes / 16,
                       (unsigned *)work);
    return hipGetLastError() == hipSuccess ? KG_OK : KG_EHIP;
}

} // extern "C"
